"""One training step of a fully connected net (config 5 and a small net) against the fp64 oracle."""
import numpy as np
import pytest

from oracle import fc as ofc
from paper_1702_03192_amd import binding as mt
from paper_1702_03192_amd import inputs as I

pytestmark = pytest.mark.gpu


def make_net(dims, batch, seed):
    X = I.normal01(seed, 0, batch, dims[0])
    labels = I.uniform_ints(seed, 1, batch, 0, dims[-1] - 1).astype(np.int32)
    W = [I.xavier_uniform(seed + 1 + l, 2, dims[l + 1], dims[l]) for l in range(len(dims) - 1)]
    b = [np.zeros(dims[l + 1], np.float32) for l in range(len(dims) - 1)]
    return X, labels, W, b


def settle_relu_decisions(X, W, b, tau=2e-4):
    """Nudge hidden-layer biases (by multiples of tau, in fp32) until every pre-activation, evaluated
    in float64 on the host, is at least tau away from zero.  The ReLU decision z > 0 is then the same
    in the kernels' fp32 as in the oracle's fp64 (the fp32 forward error is ~1e-5 at these sizes), so
    both sides take every decision identically and the comparison measures rounding, not flipped
    units.  Uses only host arithmetic on the seeded inputs.  Returns (biases, number of biases moved)."""
    moved = 0
    H = X.astype(np.float64)
    for l in range(len(W) - 1):
        zw = H @ W[l].astype(np.float64).T
        for _ in range(3):
            z = zw + b[l].astype(np.float64)
            bad = np.where(np.abs(z).min(axis=0) < tau)[0]
            if bad.size == 0:
                break
            for j in bad:
                col = z[:, j]
                for c in range(1, 400):
                    done = False
                    for sign in (1.0, -1.0):
                        d = sign * c * tau
                        if np.abs(col + d).min() >= 1.5 * tau:
                            b[l][j] = np.float32(b[l][j] + d)
                            moved += 1
                            done = True
                            break
                    if done:
                        break
        z = zw + b[l].astype(np.float64)
        assert np.abs(z).min() >= tau, "could not separate the pre-activations from zero"
        H = np.maximum(z, 0.0)
    return b, moved


def run_step(dims, batch, X, labels, W, b, lr, mode):
    import torch
    L = len(dims) - 1
    dX = torch.from_numpy(X).cuda()
    dl = torch.from_numpy(labels).cuda()
    dW_ = [torch.from_numpy(w.copy()).cuda() for w in W]
    db_ = [torch.from_numpy(v.copy()).cuda() for v in b]
    gW = [torch.full_like(w, float("nan")) for w in dW_]
    gb = [torch.full_like(v, float("nan")) for v in db_]
    loss = torch.full((1,), float("nan"), device="cuda")
    logits = torch.empty((batch, dims[-1]), device="cuda")
    ws = torch.empty(mt.mtnn_fc_workspace_bytes(dims, batch), dtype=torch.uint8, device="cuda")
    desc, keep = mt.make_fc_desc(dims, batch, dX, dl, dW_, db_, gW, gb, loss, ws, lr, mode, logits)
    mt.mtnn_fc_train_step(desc)
    torch.cuda.synchronize()
    return {"loss": float(loss.item()), "logits": logits.cpu().numpy(),
            "dW": [g.cpu().numpy() for g in gW], "db": [g.cpu().numpy() for g in gb],
            "W_new": [w.cpu().numpy() for w in dW_], "b_new": [v.cpu().numpy() for v in db_]}


def nrm_err(got, want):
    want = np.asarray(want, dtype=np.float64)
    return float(np.linalg.norm(got.astype(np.float64) - want) / max(np.linalg.norm(want), 1e-300))


def running_bounds(X, labels, W, b, ref):
    """First-order running error bounds, element by element, for a step computed in fp32 with every
    product inside 1e-5 sqrt(k) of the componentwise bound S = |A||B| (the benchmark's tolerance) and
    every ReLU decision as in `ref`: the error of a product's result is its own rounding plus the
    errors of its operands carried through it.  Host fp64 arithmetic on the oracle's intermediates;
    nothing here is part of the method."""
    from gpu_util import tol as gemm_tol
    u = 2.0 ** -24
    L = len(W)
    aW = [np.abs(w.astype(np.float64)) for w in W]
    H = ref["H"]                                   # H[0] = X, H[l] = layer l's output (post-ReLU; logits last)
    EH = [np.zeros_like(H[0])]
    for l in range(L):
        k = W[l].shape[1]
        S = np.abs(H[l]) @ aW[l].T + np.abs(b[l].astype(np.float64))
        EH.append(gemm_tol(k) * S + EH[l] @ aW[l].T + 2 * u * np.abs(H[l + 1]))      # (the clamp is 1-Lipschitz)
    batch = X.shape[0]
    p = np.exp(ref["logits"] - ref["logits"].max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    # softmax: |dp_j| <= p_j (|dz_j| + sum_i p_i |dz_i|) <= 2 p_j max_i |dz_i|; plus the kernel's own exp / log rounding
    EdZ = (2.0 * p * EH[L].max(1, keepdims=True) + 64 * u * (p + 1e-30)) / batch
    EdW, Edb = [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        dZ = ref["dZ"][l]                          # gradient w.r.t. layer l's pre-activation, batch x d_{l+1}
        EdW[l] = gemm_tol(batch) * (np.abs(dZ).T @ np.abs(H[l])) + EdZ.T @ np.abs(H[l]) + np.abs(dZ).T @ EH[l]
        Edb[l] = batch * u * np.abs(dZ).sum(0) + EdZ.sum(0)
        if l > 0:
            k = W[l].shape[0]
            EdH = gemm_tol(k) * (np.abs(dZ) @ aW[l]) + EdZ @ aW[l]
            EdZ = EdH * (H[l] > 0.0)
    return {"logits": EH[L], "dW": EdW, "db": Edb}


_REF_CACHE = {}


def check_step(dims, batch, seed, mode, lr=0.01, tol=1e-4):
    key = (tuple(dims), batch, seed, lr)
    if key not in _REF_CACHE:
        X, labels, W, b = make_net(dims, batch, seed)
        if len(dims) > 2:
            b[0] = (I.uniform_pm1(seed, 7, 1, dims[1])[0] * 0.1).astype(np.float32)   # a non-zero bias somewhere
        stated = [v.copy() for v in b]
        b, moved = settle_relu_decisions(X, W, b)
        hidden = sum(dims[1:-1])
        shift = max(float(np.abs(v - s).max()) for v, s in zip(b, stated))
        print(f"[fc inputs] dims={dims} batch={batch}: {moved} of {hidden} hidden biases moved off a ReLU threshold, "
              f"by at most {shift:.1e}")
        # (with a mini-batch of 1024 a column of pre-activations comes within 2e-4 of zero about one time in three,
        #  so many biases move -- each by a few multiples of 2e-4 only; the stated inputs themselves, biases zero,
        #  are checked product by product in test_config5_step_product_by_product_on_the_stated_inputs)
        assert moved <= hidden // 2 and shift <= 1e-2
        ref = ofc.fc_step(X, labels, W, b, lr)
        _REF_CACHE.clear()                                        # (one net at a time: the large ones are GBs)
        _REF_CACHE[key] = (X, labels, W, b, ref, running_bounds(X, labels, W, b, ref))
    X, labels, W, b, ref, bounds = _REF_CACHE[key]
    got = run_step(dims, batch, X, labels, W, b, lr, mode)
    assert abs(got["loss"] - ref["loss"]) <= 1e-5 * max(1.0, abs(ref["loss"]))
    assert nrm_err(got["logits"], ref["logits"]) <= tol
    # element by element: every logit, every weight gradient, every bias gradient inside its running bound
    excess = np.abs(got["logits"].astype(np.float64) - ref["logits"]) - bounds["logits"]
    assert (excess <= 0).all(), f"logits: {int((excess > 0).sum())} elements outside their bound, worst by {excess.max():.3g}"
    for l in range(len(dims) - 1):
        assert nrm_err(got["dW"][l], ref["dW"][l]) <= tol, f"dW[{l}]"
        assert nrm_err(got["db"][l], ref["db"][l]) <= tol, f"db[{l}]"
        assert nrm_err(got["W_new"][l], ref["W_new"][l]) <= 1e-6, f"W_new[{l}]"
        assert nrm_err(got["b_new"][l] + 1.0, ref["b_new"][l] + 1.0) <= 1e-6, f"b_new[{l}]"
        for name in ("dW", "db"):
            excess = np.abs(got[name][l].astype(np.float64) - ref[name][l]) - bounds[name][l]
            assert (excess <= 0).all(), \
                f"{name}[{l}]: {int((excess > 0).sum())} elements outside their bound, worst by {excess.max():.3g}"
        # the update itself, element by element: W_new = W - lr dW with the GPU's own dW, to one rounding
        want_w = W[l].astype(np.float64) - float(np.float32(lr)) * got["dW"][l].astype(np.float64)
        assert (np.abs(got["W_new"][l].astype(np.float64) - want_w) <= 2.0 ** -23 * np.abs(want_w) + 1e-30).all(), f"W_new[{l}]"
        want_b = b[l].astype(np.float64) - float(np.float32(lr)) * got["db"][l].astype(np.float64)
        assert (np.abs(got["b_new"][l].astype(np.float64) - want_b) <= 2.0 ** -23 * np.abs(want_b) + 1e-30).all(), f"b_new[{l}]"
    return got


@pytest.mark.parametrize("mode", [0, 1, -1], ids=["auto", "nt", "tnn"])
def test_small_net_all_forward_modes(mode):
    check_step([37, 70, 45, 10], 33, 5100, mode)


def test_forward_modes_agree_and_rerun_is_bit_identical():
    dims, batch = [100, 200, 150, 10], 64
    X, labels, W, b = make_net(dims, batch, 5200)
    a = run_step(dims, batch, X, labels, W, b, 0.01, 1)
    a2 = run_step(dims, batch, X, labels, W, b, 0.01, 1)
    t = run_step(dims, batch, X, labels, W, b, 0.01, -1)
    assert a["loss"] == a2["loss"]
    for l in range(3):
        assert a["W_new"][l].tobytes() == a2["W_new"][l].tobytes()
        assert nrm_err(a["dW"][l], t["dW"][l]) < 1e-5


@pytest.mark.parametrize("mode", [1, -1, 0], ids=["nt", "tnn", "auto"])
def test_config5_step(mode):
    cfg = I.CONFIG5
    check_step(cfg["dims"], cfg["batch"], cfg["seed"], mode)


@pytest.mark.parametrize("batch,width", [(50, 72), (1000, 200), (1024, 4096), (33, 8)])
def test_elementwise_16_byte_paths_against_numpy(batch, width):
    """Widths that are multiples of 4 take the 16-byte kernels: bias + ReLU, ReLU mask with the bias
    gradient in the same pass (with and without scratch), SGD."""
    import torch
    z = I.normal01(5310, 0, batch, width)
    bias = I.normal01(5310, 1, 1, width)[0]
    g = I.normal01(5310, 2, batch, width)
    for relu in (True, False):
        Z = torch.from_numpy(z.copy()).cuda()
        mt.mtnn_fc_bias_act(Z, torch.from_numpy(bias).cuda(), relu)
        want = z + bias
        assert np.array_equal(Z.cpu().numpy(), np.maximum(want, np.float32(0)) if relu else want)
    H = np.maximum(z, np.float32(0))
    masked = np.where(H > 0, g, np.float32(0))
    want_db = masked.astype(np.float64).sum(0)
    # fp32 summation in any order: |error| <= (rows - 1) 2^-24 sum |x| per column
    tol_db = batch * 2.0 ** -24 * np.abs(masked).astype(np.float64).sum(0).max()
    for scratch in (torch.empty(32 * width, device="cuda"), None):
        dH = torch.from_numpy(g.copy()).cuda()
        db = torch.full((width,), float("nan"), device="cuda")
        mt.mtnn_fc_relu_backward_bias_grad(dH, torch.from_numpy(H).cuda(), db, scratch)
        assert np.array_equal(dH.cpu().numpy(), masked)
        assert np.abs(db.cpu().numpy() - want_db).max() <= tol_db
        db2 = torch.full((width,), float("nan"), device="cuda")
        mt.mtnn_fc_bias_grad(dH, db2, scratch)
        assert np.abs(db2.cpu().numpy() - want_db).max() <= tol_db
    P = torch.from_numpy(z.copy()).cuda()
    mt.mtnn_fc_sgd(P, torch.from_numpy(g).cuda(), 0.25)
    assert np.array_equal(P.cpu().numpy(), z - np.float32(0.25) * g)


def test_elementwise_steps_against_numpy():
    import torch
    rng_z = I.normal01(5300, 0, 50, 70)
    bias = I.normal01(5300, 1, 1, 70)[0]
    Z = torch.from_numpy(rng_z.copy()).cuda()
    mt.mtnn_fc_bias_act(Z, torch.from_numpy(bias).cuda(), True)
    assert np.array_equal(Z.cpu().numpy(), np.maximum(rng_z + bias, np.float32(0)))
    Z2 = torch.from_numpy(rng_z.copy()).cuda()
    mt.mtnn_fc_bias_act(Z2, torch.from_numpy(bias).cuda(), False)
    assert np.array_equal(Z2.cpu().numpy(), rng_z + bias)
    # relu backward
    H = torch.from_numpy(np.maximum(rng_z, 0)).cuda()
    dH = torch.from_numpy(bias[None, :].repeat(50, 0).copy()).cuda()
    mt.mtnn_fc_relu_backward(dH, H)
    assert np.array_equal(dH.cpu().numpy(), np.where(rng_z > 0, bias[None, :], np.float32(0)))
    # bias gradient (column sums)
    dZ = torch.from_numpy(rng_z.copy()).cuda()
    db = torch.empty(70, device="cuda")
    mt.mtnn_fc_bias_grad(dZ, db)
    assert np.allclose(db.cpu().numpy(), rng_z.astype(np.float64).sum(0), rtol=1e-5, atol=1e-5)
    big = I.normal01(5301, 0, 1000, 200)
    dbig = torch.from_numpy(big).cuda()
    db2 = torch.empty(200, device="cuda")
    db3 = torch.empty(200, device="cuda")
    mt.mtnn_fc_bias_grad(dbig, db2, scratch=torch.empty(32 * 200, device="cuda"))
    mt.mtnn_fc_bias_grad(dbig, db3)
    want = big.astype(np.float64).sum(0)
    assert np.allclose(db2.cpu().numpy(), want, rtol=1e-5, atol=1e-4)
    assert np.allclose(db3.cpu().numpy(), want, rtol=1e-5, atol=1e-4)
    # sgd
    P = torch.from_numpy(rng_z.copy()).cuda()
    mt.mtnn_fc_sgd(P, dZ, 0.5)
    assert np.array_equal(P.cpu().numpy(), rng_z - np.float32(0.5) * rng_z)
    # softmax cross-entropy
    labels = I.uniform_ints(5300, 2, 50, 0, 69).astype(np.int32)
    out = torch.empty((50, 70), device="cuda")
    rl = torch.empty(50, device="cuda")
    ml = torch.empty(1, device="cuda")
    mt.mtnn_fc_softmax_xent(torch.from_numpy(rng_z).cuda(), torch.from_numpy(labels).cuda(), out, rl, ml)
    torch.cuda.synchronize()
    z = rng_z.astype(np.float64)
    lp = z - z.max(1, keepdims=True)
    lp = lp - np.log(np.exp(lp).sum(1, keepdims=True))
    want = np.exp(lp)
    want[np.arange(50), labels] -= 1
    assert np.allclose(out.cpu().numpy(), want / 50, rtol=1e-5, atol=1e-7)
    assert np.allclose(rl.cpu().numpy(), -lp[np.arange(50), labels], rtol=1e-5, atol=1e-6)
    assert abs(ml.item() + lp[np.arange(50), labels].mean()) < 1e-5


@pytest.mark.parametrize("dims,batch", [([784, 2048, 1024, 10], 128), ([784, 2048, 2048, 2048, 1024, 10], 64)],
                         ids=["mnist-2-hidden", "mnist-4-hidden"])
def test_table_ix_mnist_sized_nets(dims, batch):
    check_step(dims, batch, 5400 + len(dims), 0)


def test_table_ix_synthetic_wide_net():
    # 26752 inputs and outputs, two hidden layers of 4096 (Table IX), a small mini-batch
    check_step([26752, 4096, 4096, 26752], 32, 5500, 0)


def test_forward_only_entry_matches_the_step_and_leaves_the_weights():
    import torch
    dims, batch = [100, 200, 150, 10], 64
    X, labels, W, b = make_net(dims, batch, 5600)
    full = run_step(dims, batch, X, labels, W, b, 0.01, 1)
    dX = torch.from_numpy(X).cuda()
    dl = torch.from_numpy(labels).cuda()
    dW_ = [torch.from_numpy(w.copy()).cuda() for w in W]
    db_ = [torch.from_numpy(v.copy()).cuda() for v in b]
    loss = torch.full((1,), float("nan"), device="cuda")
    logits = torch.empty((batch, dims[-1]), device="cuda")
    ws = torch.empty(mt.mtnn_fc_workspace_bytes(dims, batch), dtype=torch.uint8, device="cuda")
    desc, keep = mt.make_fc_desc(dims, batch, dX, dl, dW_, db_, dW_, db_, loss, ws, 0.01, 1, logits)
    mt.mtnn_fc_forward(desc)
    torch.cuda.synchronize()
    assert float(loss.item()) == full["loss"]
    assert logits.cpu().numpy().tobytes() == full["logits"].tobytes()
    for l in range(3):
        assert dW_[l].cpu().numpy().tobytes() == W[l].tobytes()


# ---- the two products with their elementwise step in the epilogue ---------------------------------

# (m, n, k, ldx pad, ldw pad, ldy pad, operands fit the pipelined kernel)
FORWARD_CASES = [
    (128, 2048, 784, 0, 0, 0, True),       # a Table IX layer at mini-batch 128: pipelined kernel
    (1024, 4096, 4096, 0, 0, 0, True),     # a config-2 shape
    (4096, 4096, 1024, 0, 0, 0, True),     # the other one: 256 x 256 tiles, whose NT columns are interleaved per lane
    (4000, 4000, 1000, 0, 0, 0, True),     # ... with ragged edge tiles
    (200, 328, 1000, 0, 0, 0, True),       # ragged tiles, operands still in 16-byte chunks
    (256, 512, 260, 4, 8, 4, True),        # padded leading dimensions (multiples of 4)
    (64, 128, 8192, 0, 0, 0, True),        # split-k: the reduction kernel carries the epilogue
    (1024, 1024, 1024, 0, 0, 0, True),     # one 64 x 64 tile per CU: the configuration with two sets of waves per workgroup
    (1000, 1000, 1000, 0, 0, 0, True),     # ... with ragged edge tiles
    (32, 8192, 4096, 0, 0, 0, True),       # one tile high: split-k over the two-wave-set 32 x 256 tile
    (100, 37, 51, 0, 0, 0, False),         # nothing aligned: guarded kernel + separate pass
    (96, 130, 64, 0, 0, 3, True),          # n % 4 != 0 with a padded Y: word-wise stores (NT); not for the NN product of TNN
    (5, 7, 0, 0, 0, 0, False),             # k = 0: Y = act(b) in every row
]


@pytest.mark.parametrize("mode", [1, -1], ids=["nt", "tnn"])
@pytest.mark.parametrize("relu", [True, False], ids=["relu", "linear"])
@pytest.mark.parametrize("case", FORWARD_CASES, ids=lambda c: "x".join(map(str, c[:3])))
def test_layer_forward_is_the_product_then_bias_then_clamp(case, relu, mode):
    """mtnn_fc_layer_forward against (a) the library's own separate calls, bit for bit, and (b) the fp64
    oracle product with the bias and clamp applied in float64, to the product's tolerance."""
    import torch
    from oracle import gemm as og
    from tests.gpu_util import Guarded, dev_matrix, tol
    m, n, k, px, pw, py, expect_fused = case
    seed = 500 + m + n + k
    A = I.uniform_pm1(seed, 0, m, max(k, 1))[:, :k]
    B = I.uniform_pm1(seed, 1, n, max(k, 1))[:, :k]
    b = (I.uniform_pm1(seed, 2, 1, n)[0] * np.float32(0.5 * np.sqrt(max(k, 1)))).astype(np.float32)
    dA = dev_matrix(np.ascontiguousarray(A), max(k + px, 1))
    dB = dev_matrix(np.ascontiguousarray(B), max(k + pw, 1))
    db = torch.from_numpy(b).cuda()
    ws = torch.empty(max(mt.mtnn_tnn_workspace_bytes(n, k), 256), dtype=torch.uint8, device="cuda")
    plain = Guarded(m, n, n + py)
    (mt.mtnn_nt if mode == 1 else lambda a_, b_, c_: mt.mtnn_tnn(a_, b_, c_, ws))(dA, dB, plain.view)
    want_bits = plain.view + db
    if relu:
        want_bits = torch.where(want_bits > 0, want_bits, torch.zeros_like(want_bits))
    out = Guarded(m, n, n + py)
    before = mt.mtnn_gemm_fused_epilogue_launches()
    chosen = mt.mtnn_fc_layer_forward(dA, dB, db, out.view, relu, mode, ws)
    torch.cuda.synchronize()
    assert chosen == mode
    if k > 0:
        # (the NN product of TNN also needs n in 16-byte chunks)
        # operands in 16-byte chunks fuse (in the kernel, or in the reduction kernel of a split-k launch),
        # unless the rule finds the even cut worth a separate pass
        want_fused = expect_fused and (mode == 1 or n % 4 == 0)
        if mt.mtnn_gemm_default_splits(mt.OP_NT if mode == 1 else mt.OP_NN, m, n, k) != mt.EVEN_CUT:
            assert (mt.mtnn_gemm_fused_epilogue_launches() == before + 1) == want_fused
    else:
        assert mt.mtnn_gemm_fused_epilogue_launches() == before
    Y, intact = out.host()
    assert intact, "wrote outside Y"
    assert np.array_equal(Y.view(np.uint32), want_bits.cpu().numpy().view(np.uint32)), "differs from the separate calls"
    if k > 0:
        C_ref, S_ref = og.nt_ref(A, B, with_bound=True)
        z = C_ref + b.astype(np.float64)
        want = np.maximum(z, 0.0) if relu else z
        # the clamp is 1-Lipschitz, so the product's componentwise bound carries over (plus one rounding of the sum)
        err = np.abs(Y.astype(np.float64) - want)
        bound = tol(k) * S_ref + 2.0 ** -23 * np.abs(z)
        assert (err <= bound).all(), f"max excess {(err - bound).max():.3g}"


def test_layer_forward_auto_mode_reports_the_selected_path():
    import torch
    m, n, k = 256, 512, 256
    A = torch.from_numpy(I.uniform_pm1(71, 0, m, k)).cuda()
    B = torch.from_numpy(I.uniform_pm1(71, 1, n, k)).cuda()
    b = torch.from_numpy(I.uniform_pm1(71, 2, 1, n)[0]).cuda()
    Y = torch.empty((m, n), device="cuda")
    ws = torch.empty(mt.mtnn_tnn_workspace_bytes(n, k), dtype=torch.uint8, device="cuda")
    assert mt.mtnn_fc_layer_forward(A, B, b, Y, True, 0, ws) == mt.mtnn_select(m, n, k)
    assert mt.mtnn_fc_layer_forward(A, B, b, Y, True, 0, None) == 1       # no room for B^T: NT (Section II)


# (m, n, k, lda pad, ldb pad, lddw pad, ldw pad, expect the fused path)
UPDATE_CASES = [
    (2048, 784, 128, 0, 0, 0, 0, True),     # dW of a Table IX layer at mini-batch 128
    (1024, 2048, 4096, 0, 0, 0, 0, True),   # ... at mini-batch 4096
    (200, 328, 260, 0, 0, 0, 0, True),      # ragged tiles
    (256, 512, 64, 4, 4, 8, 4, True),       # padded leading dimensions
    (10, 1024, 4096, 0, 0, 0, 0, True),     # small m n, long k: fused only if the rule does not split it
    (1024, 1024, 1024, 0, 0, 0, 0, True),   # one 64 x 64 tile per CU: two sets of waves per workgroup, update in set 0's epilogue
    (4096, 4096, 1024, 0, 0, 0, 0, True),   # config 5's weight gradients (the plain product would take the 16-wide-slab configuration)
    (100, 37, 51, 0, 0, 0, 0, False),       # unaligned: separate pass
    (64, 128, 96, 0, 0, 0, 3, None),        # W rows not 16-byte aligned: fused kernel, word-wise update
]


@pytest.mark.parametrize("case", UPDATE_CASES, ids=lambda c: "x".join(map(str, c[:3])))
def test_weight_grad_sgd_is_the_product_then_the_update(case):
    """mtnn_fc_weight_grad_sgd against mtnn_nn followed by mtnn_fc_sgd, bit for bit, and against the fp64
    oracle (dW to the product's tolerance; W to that times lr plus one rounding)."""
    import torch
    from oracle import gemm as og
    from tests.gpu_util import Guarded, dev_matrix, tol
    m, n, k, pa, pb, pg, pw, expect_fused = case
    lr = np.float32(0.05)
    seed = 900 + m + n + k
    A = I.uniform_pm1(seed, 0, m, k)
    B = I.uniform_pm1(seed, 1, k, n)
    W0 = I.uniform_pm1(seed, 2, m, n)
    dA, dB = dev_matrix(A, k + pa), dev_matrix(B, n + pb)
    # reference: the separate calls (dense W, as mtnn_fc_sgd wants it)
    g_ref = torch.empty((m, n), device="cuda")
    w_ref = torch.from_numpy(W0.copy()).cuda()
    mt.mtnn_nn(dA, dB, g_ref)
    mt.mtnn_fc_sgd(w_ref, g_ref, float(lr))
    g = Guarded(m, n, n + pg)
    w = Guarded(m, n, n + pw)
    w.view.copy_(torch.from_numpy(W0).cuda())
    before = mt.mtnn_gemm_fused_epilogue_launches()
    mt.mtnn_fc_weight_grad_sgd(dA, dB, g.view, w.view, float(lr))
    torch.cuda.synchronize()
    if expect_fused is not None and mt.mtnn_gemm_default_splits(mt.OP_NN, m, n, k) == 1:
        # (a weight gradient the rule splits over k updates in a separate pass)
        assert (mt.mtnn_gemm_fused_epilogue_launches() == before + 1) == expect_fused
    G, ok_g = g.host()
    Wn, ok_w = w.host()
    assert ok_g and ok_w, "wrote outside dW or W"
    assert np.array_equal(G.view(np.uint32), g_ref.cpu().numpy().view(np.uint32)), "dW differs from mtnn_nn"
    assert np.array_equal(Wn.view(np.uint32), w_ref.cpu().numpy().view(np.uint32)), "W differs from the separate update"
    C_ref, S_ref = og.nn_ref(A, B, with_bound=True)
    assert (np.abs(G.astype(np.float64) - C_ref) <= tol(k) * S_ref).all()
    want_w = W0.astype(np.float64) - float(lr) * C_ref
    bound = float(lr) * tol(k) * S_ref + 2.0 ** -23 * np.abs(want_w) + 1e-30
    assert (np.abs(Wn.astype(np.float64) - want_w) <= bound).all()


def test_step_uses_the_fused_epilogues():
    """A step of an aligned net runs every forward product and every weight gradient with its epilogue fused."""
    dims, batch = [784, 2048, 1024, 10], 128
    X, labels, W, b = make_net(dims, batch, 31)
    before = mt.mtnn_gemm_fused_epilogue_launches()
    run_step(dims, batch, X, labels, W, b, 0.01, 1)
    # 3 forward products; of the 3 weight gradients the 10 x 1024 one may be split over k (then it updates separately)
    assert mt.mtnn_gemm_fused_epilogue_launches() - before >= 5


def test_step_is_bit_identical_with_and_without_fused_epilogues():
    """The process-wide switch turns every fused epilogue into the plain product plus its separate pass;
    logits, loss, gradients and updated parameters of a step must not change by a bit."""
    dims, batch = [784, 2048, 1024, 10], 256
    X, labels, W, b = make_net(dims, batch, 77)
    b[0] = (I.uniform_pm1(77, 7, 1, dims[1])[0] * 0.1).astype(np.float32)
    fused = run_step(dims, batch, X, labels, W, b, 0.05, 1)
    assert mt.mtnn_set_fused_epilogues(False) is True
    try:
        before = mt.mtnn_gemm_fused_epilogue_launches()
        plain = run_step(dims, batch, X, labels, W, b, 0.05, 1)
        assert mt.mtnn_gemm_fused_epilogue_launches() == before
    finally:
        assert mt.mtnn_set_fused_epilogues(True) is False
    assert fused["loss"] == plain["loss"]
    assert np.array_equal(fused["logits"].view(np.uint32), plain["logits"].view(np.uint32))
    for key in ("dW", "db", "W_new", "b_new"):
        for l, (x, y) in enumerate(zip(fused[key], plain[key])):
            assert np.array_equal(x.view(np.uint32), y.view(np.uint32)), f"{key}[{l}] differs"


# ---- the step product by product, each product checked on the inputs it really had -----------------

def _host(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy().copy()


def composed_step(dims, batch, X, labels, W, b, lr, mode, check):
    """The training step put together from the library's exported pieces in the order
    mtnn_fc_train_step issues them, with every intermediate copied to the host.  `check(kind, ...)` is
    called for every product, transpose and elementwise pass with the values that pass really read and
    wrote.  Returns the same dict as run_step."""
    import torch
    L = len(dims) - 1
    max_w = max(dims)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    dW_ = [dev(w.copy()) for w in W]
    db_ = [dev(v.copy()) for v in b]
    gW = [torch.full_like(w, float("nan")) for w in dW_]
    gb = [torch.full_like(v, float("nan")) for v in db_]
    H = [dev(X)] + [torch.full((batch, dims[l + 1]), float("nan"), device="cuda") for l in range(L)]
    dl = dev(labels)
    bt_ws = torch.empty(max(mt.mtnn_tnn_workspace_bytes(dims[l + 1], dims[l]) for l in range(L)), dtype=torch.uint8, device="cuda")
    bias_part = torch.empty(32 * max_w, device="cuda")
    row_loss = torch.empty(batch, device="cuda")
    loss = torch.full((1,), float("nan"), device="cuda")
    lr32 = float(np.float32(lr))
    for l in range(L):
        h_in = _host(H[l])
        chosen = mt.mtnn_fc_layer_forward(H[l], dW_[l], db_[l], H[l + 1], relu=(l < L - 1), mode=mode, workspace=bt_ws)
        check("forward", l, h_in, W[l], b[l], _host(H[l + 1]), l < L - 1, chosen)
    logits = _host(H[L])
    dZ = torch.full((batch, dims[L]), float("nan"), device="cuda")
    mt.mtnn_fc_softmax_xent(H[L], dl, dZ, row_loss, loss)
    check("softmax", logits, labels, _host(dZ), _host(row_loss), float(_host(loss)[0]))
    for l in range(L - 1, -1, -1):
        fan_in, fan_out = dims[l], dims[l + 1]
        dz_host = _host(dZ)
        if l == L - 1:
            mt.mtnn_fc_bias_grad(dZ, gb[l], bias_part)
            check("bias_grad", l, dz_host, _host(gb[l]))
            mt.mtnn_fc_sgd(db_[l], gb[l], lr32)
        if l > 0:
            dNext = torch.full((batch, fan_in), float("nan"), device="cuda")
            mt.mtnn_nn(dZ, dW_[l], dNext)                                    # (the weights before their update)
            dh_host = _host(dNext)
            check("input_grad", l, dz_host, W[l], dh_host)
            mt.mtnn_fc_relu_backward_bias_grad(dNext, H[l], gb[l - 1], bias_part)
            check("mask_bias_grad", l - 1, dh_host, _host(H[l]), _host(dNext), _host(gb[l - 1]))
            mt.mtnn_fc_sgd(db_[l - 1], gb[l - 1], lr32)
        dZt = torch.full((fan_out, batch), float("nan"), device="cuda")
        mt.mtnn_transpose(dZ, dZt)
        dzt_host = _host(dZt)
        check("transpose", l, dz_host, dzt_host)
        h_host = _host(H[l])
        mt.mtnn_fc_weight_grad_sgd(dZt, H[l], gW[l], dW_[l], lr32)
        check("weight_grad", l, dzt_host, h_host, W[l], _host(gW[l]), _host(dW_[l]), lr32)
        if l > 0:
            dZ = dNext
    torch.cuda.synchronize()
    return {"loss": float(loss.item()), "logits": logits,
            "dW": [g.cpu().numpy() for g in gW], "db": [g.cpu().numpy() for g in gb],
            "W_new": [w.cpu().numpy() for w in dW_], "b_new": [v.cpu().numpy() for v in db_]}


def product_checker(log):
    """check() for composed_step: every product against the oracle's product of the SAME fp32 inputs, element
    by element at 1e-5 sqrt(k) of S; transposes and masks bit for bit; reductions inside their fp32 bounds."""
    import oracle
    from gpu_util import tol as gemm_tol
    u = 2.0 ** -24

    def check(kind, *a):
        if kind == "forward":
            l, h_in, w, bias, h_out, relu, chosen = a
            k = w.shape[1]
            C, S = oracle.nt_ref(h_in, w, with_bound=True)
            z = C + bias.astype(np.float64)
            want = np.maximum(z, 0.0) if relu else z
            # the clamp is 1-Lipschitz: whichever side of zero the fp32 pre-activation fell, the output is within
            # the product's bound of max(z, 0); plus one rounding of the bias addition
            excess = np.abs(h_out.astype(np.float64) - want) - (gemm_tol(k) * S + 2 * u * np.abs(z))
            assert (excess <= 0).all(), f"forward product of layer {l}: {int((excess > 0).sum())} elements out, worst {excess.max():.3g}"
            log.append(("forward", l, chosen, float((np.abs(h_out - want) / np.where(S > 0, S, 1)).max())))
        elif kind == "input_grad":
            l, dz, w, dh = a
            k = w.shape[0]
            C, S = oracle.nn_ref(dz, w, with_bound=True)
            excess = np.abs(dh.astype(np.float64) - C) - gemm_tol(k) * S
            assert (excess <= 0).all(), f"input-gradient product of layer {l}: worst excess {excess.max():.3g}"
            log.append(("input_grad", l, float((np.abs(dh - C) / np.where(S > 0, S, 1)).max())))
        elif kind == "weight_grad":
            l, dzt, h, w_old, gw, w_new, lr = a
            k = dzt.shape[1]
            C, S = oracle.nn_ref(dzt, h, with_bound=True)
            excess = np.abs(gw.astype(np.float64) - C) - gemm_tol(k) * S
            assert (excess <= 0).all(), f"weight-gradient product of layer {l}: worst excess {excess.max():.3g}"
            want_w = w_old.astype(np.float64) - lr * gw.astype(np.float64)
            assert (np.abs(w_new.astype(np.float64) - want_w) <= 2 * u * np.abs(want_w) + 1e-30).all(), f"update of W[{l}]"
            log.append(("weight_grad", l, float((np.abs(gw - C) / np.where(S > 0, S, 1)).max())))
        elif kind == "transpose":
            l, dz, dzt = a
            assert dzt.tobytes() == np.ascontiguousarray(oracle.transpose_ref(dz)).tobytes(), f"transpose of dZ[{l}]"
        elif kind == "mask_bias_grad":
            l, dh, h, masked, gb = a
            want = np.where(h > 0, dh, np.float32(0))
            assert masked.tobytes() == want.tobytes(), f"ReLU mask of layer {l}"
            sums = want.astype(np.float64).sum(0)
            assert (np.abs(gb - sums) <= want.shape[0] * u * np.abs(want).astype(np.float64).sum(0) + 1e-30).all(), f"db[{l}]"
        elif kind == "bias_grad":
            l, dz, gb = a
            sums = dz.astype(np.float64).sum(0)
            assert (np.abs(gb - sums) <= dz.shape[0] * u * np.abs(dz).astype(np.float64).sum(0) + 1e-30).all(), f"db[{l}]"
        elif kind == "softmax":
            logits, labels, dz, row_loss, loss = a
            z = logits.astype(np.float64)
            lp = z - z.max(1, keepdims=True)
            lp = lp - np.log(np.exp(lp).sum(1, keepdims=True))
            want = np.exp(lp)
            want[np.arange(len(labels)), labels] -= 1.0
            want /= len(labels)
            assert np.allclose(dz, want, rtol=2e-5, atol=1e-9)
            assert np.allclose(row_loss, -lp[np.arange(len(labels)), labels], rtol=1e-5, atol=1e-6)
            assert abs(loss + lp[np.arange(len(labels)), labels].mean()) <= 1e-5
    return check


@pytest.mark.parametrize("mode", [1, -1], ids=["nt", "tnn"])
def test_config5_step_product_by_product_on_the_stated_inputs(mode):
    """Config 5 exactly as stated (biases zero, nothing nudged): the step assembled from the exported
    pieces, every product checked element-wise against the oracle on the inputs that product really
    read, and the assembled step equal, bit for bit, to mtnn_fc_train_step on the same inputs.  Comparing
    product by product needs no agreement between fp32 and fp64 ReLU decisions."""
    cfg = I.CONFIG5
    dims, batch = cfg["dims"], cfg["batch"]
    X, labels, W, b = make_net(dims, batch, cfg["seed"])
    assert all(not v.any() for v in b)
    log = []
    pieces = composed_step(dims, batch, X, labels, W, b, 0.01, mode, product_checker(log))
    assert sum(1 for e in log if e[0] == "forward") == 4 and sum(1 for e in log if e[0] == "weight_grad") == 4
    assert sum(1 for e in log if e[0] == "input_grad") == 3
    assert all(e[2] == mode for e in log if e[0] == "forward")
    whole = run_step(dims, batch, X, labels, W, b, 0.01, mode)
    assert whole["loss"] == pieces["loss"]
    assert whole["logits"].tobytes() == pieces["logits"].tobytes()
    for key in ("dW", "db", "W_new", "b_new"):
        for l, (x, y) in enumerate(zip(whole[key], pieces[key])):
            assert x.tobytes() == y.tobytes(), f"{key}[{l}]: the step differs from its pieces"


def test_small_ragged_net_product_by_product_auto_mode():
    dims, batch = [37, 70, 45, 10], 33
    X, labels, W, b = make_net(dims, batch, 5100)
    b[0] = (I.uniform_pm1(5100, 7, 1, dims[1])[0] * 0.1).astype(np.float32)
    log = []
    pieces = composed_step(dims, batch, X, labels, W, b, 0.05, 0, product_checker(log))
    whole = run_step(dims, batch, X, labels, W, b, 0.05, 0)
    assert whole["loss"] == pieces["loss"] and whole["logits"].tobytes() == pieces["logits"].tobytes()
    for key in ("dW", "db", "W_new", "b_new"):
        for l, (x, y) in enumerate(zip(whole[key], pieces[key])):
            assert x.tobytes() == y.tobytes(), f"{key}[{l}]: the step differs from its pieces"
