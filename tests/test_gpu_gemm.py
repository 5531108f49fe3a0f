"""mtnn_nt / mtnn_nn / mtnn_tnn / mtnn_auto against the fp64 CPU oracle.

Tolerance (the benchmark's definition): max relative error <= 1e-5 * sqrt(k), read both
componentwise against S = |A| |B|^T and normwise against max |C| (see gpu_util.check_gemm).
Integer-valued inputs must match bit for bit.
"""
import numpy as np
import pytest

import oracle
from paper_1702_03192_amd import binding as mt
from paper_1702_03192_amd import inputs as I
from gpu_util import Guarded, check_gemm, dev_matrix

pytestmark = pytest.mark.gpu

NCFG = 16


def sync():
    import torch
    torch.cuda.synchronize()


def run(op, cfg, A, B, lda=None, ldb=None, ldc=None, misalign=0, splits=0):
    """Run one GEMM through the C ABI; returns the fp32 host result (guard bands verified)."""
    m, k = A.shape
    n = B.shape[0] if op == mt.OP_NT else B.shape[1]
    dA, dB = dev_matrix(A, lda, misalign=misalign), dev_matrix(B, ldb, misalign=2 * misalign)
    out = Guarded(m, n, ldc, misalign=misalign)
    mt.mtnn_gemm_ex(op, cfg, dA, dB, out.view, splits=splits)
    sync()
    got, intact = out.host()
    assert intact, "GEMM wrote outside its logical output"
    return got


def reference(op, A, B, rows=None):
    return (oracle.nt_ref if op == mt.OP_NT else oracle.nn_ref)(A, B, rows=rows, with_bound=True)


def operands(op, m, n, k, seed, dist="uniform"):
    A, B = I.nt_operands(m, n, k, seed, dist)
    if op == mt.OP_NN:
        B = np.ascontiguousarray(B.T)          # k x n
    return A, B


def test_config_count_matches():
    assert len(mt.gemm_configs()) == NCFG


@pytest.mark.parametrize("op", [mt.OP_NT, mt.OP_NN], ids=["NT", "NN"])
@pytest.mark.parametrize("cfg", list(range(NCFG)))
@pytest.mark.parametrize("m,n,k", [(300, 520, 77), (64, 64, 64), (33, 31, 5), (257, 255, 130), (130, 260, 100),
                                   (70, 36, 12), (264, 392, 200)])
def test_every_config_against_oracle(op, cfg, m, n, k):
    A, B = operands(op, m, n, k, 100 + cfg)
    got = run(op, cfg, A, B)
    C, S = reference(op, A, B)
    check_gemm(got, C, S, k, f"op{op} cfg{cfg} {m}x{n}x{k}")


@pytest.mark.parametrize("op", [mt.OP_NT, mt.OP_NN], ids=["NT", "NN"])
@pytest.mark.parametrize("cfg", list(range(NCFG)))
def test_integer_inputs_are_bit_exact(op, cfg):
    m, n, k = 290, 275, 203
    A, B = operands(op, m, n, k, 200 + cfg, dist="int")
    got = run(op, cfg, A, B)
    C, _ = reference(op, A, B)
    assert np.array_equal(got, C.astype(np.float32))


@pytest.mark.parametrize("op", [mt.OP_NT, mt.OP_NN], ids=["NT", "NN"])
@pytest.mark.parametrize("cfg", [-1, 0, 1, 4, 5])
def test_odd_leading_dimensions_nan_padding_and_misaligned_bases(op, cfg):
    m, n, k = 131, 262, 45
    A, B = operands(op, m, n, k, 300)
    C, S = reference(op, A, B)
    bcols = B.shape[1]
    for (lda, ldb, ldc, mis) in [(k + 3, bcols + 3, n + 3, 0), (k + 4, bcols + 8, n + 1, 0), (k, bcols, n, 1)]:
        got = run(op, cfg, A, B, lda, ldb, ldc, misalign=mis)       # padding holds NaN
        check_gemm(got, C, S, k, f"op{op} cfg{cfg} ld+({lda - k},{ldb - bcols},{ldc - n})")


@pytest.mark.parametrize("op", [mt.OP_NT, mt.OP_NN], ids=["NT", "NN"])
@pytest.mark.parametrize("k", [1, 2, 3, 4, 7, 8, 9, 15, 16, 17, 31, 33])
def test_k_tails(op, k):
    m, n = 70, 90
    A, B = operands(op, m, n, k, 400 + k, dist="normal")
    got = run(op, -1, A, B)
    C, S = reference(op, A, B)
    check_gemm(got, C, S, k, f"op{op} k={k}")


@pytest.mark.parametrize("op", [mt.OP_NT, mt.OP_NN], ids=["NT", "NN"])
@pytest.mark.parametrize("cfg,splits", [(0, 2), (2, 3), (3, 4), (3, 32), (4, 5), (5, 8), (-1, 0), (1, 16)])
@pytest.mark.parametrize("m,n,k", [(70, 92, 1000), (300, 264, 2052), (33, 520, 4099)])
def test_split_k_against_oracle(op, cfg, splits, m, n, k):
    A, B = operands(op, m, n, k, 600 + splits, dist="normal")
    got = run(op, cfg, A, B, splits=splits)
    C, S = reference(op, A, B)
    check_gemm(got, C, S, k, f"op{op} cfg{cfg} splits{splits} {m}x{n}x{k}")
    again = run(op, cfg, A, B, splits=splits)
    assert again.tobytes() == got.tobytes()            # fixed reduction order


def test_split_k_integer_inputs_bit_exact_and_padding():
    m, n, k = 100, 136, 1536
    for op in (mt.OP_NT, mt.OP_NN):
        A, B = operands(op, m, n, k, 650, dist="int")
        C, _ = reference(op, A, B)
        got = run(op, 3, A, B, ldc=n + 5, splits=6)
        assert np.array_equal(got, C.astype(np.float32))


def test_degenerate_sizes():
    import torch
    out = Guarded(6, 9, 11)
    a = torch.zeros((6, 1), device="cuda")
    b = torch.zeros((9, 1), device="cuda")
    L = mt.lib()
    # k == 0: the empty sum
    assert L.mtnn_nt(None, 6, 9, 0, None, 1, None, 1, out.view.data_ptr(), 11) == 0
    sync()
    got, intact = out.host()
    assert intact and np.array_equal(got, np.zeros((6, 9), np.float32)) and not np.signbit(got).any()
    out2 = Guarded(6, 9)
    assert L.mtnn_nn(None, 0, 9, 4, a.data_ptr(), 4, b.data_ptr(), 9, out2.view.data_ptr(), 9) == 0
    assert L.mtnn_nt(None, 6, 0, 4, a.data_ptr(), 4, b.data_ptr(), 4, out2.view.data_ptr(), 1) == 0
    sync()
    assert np.isnan(out2.host()[0]).all()          # untouched


def test_identity_and_permutation_on_device():
    A = I.uniform_pm1(500, 0, 100, 96)
    eye = np.eye(96, dtype=np.float32)
    assert np.array_equal(run(mt.OP_NT, -1, A, eye), A)
    assert np.array_equal(run(mt.OP_NN, -1, A, eye), A)
    perm = I.uniform_ints(501, 0, 96, 0, 10 ** 6).argsort()
    assert np.array_equal(run(mt.OP_NT, -1, A, eye[perm]), A[:, perm])


# ---- the benchmark configurations -----------------------------------------------------------

def check_all_paths(m, n, k, seed, dist, rows=None):
    """NT, TNN and auto on one shape against the oracle (all rows, or a row sample)."""
    import torch
    A, B = I.nt_operands(m, n, k, seed, dist)
    C, S = oracle.nt_ref(A, B, rows=rows, with_bound=True)
    dA, dB = dev_matrix(A), dev_matrix(B)
    ws = torch.empty(mt.mtnn_tnn_workspace_bytes(n, k), dtype=torch.uint8, device="cuda")
    pick = (lambda x: x) if rows is None else (lambda x: x[rows])
    outs = {}
    for name in ("nt", "tnn", "auto"):
        out = Guarded(m, n)
        if name == "nt":
            mt.mtnn_nt(dA, dB, out.view)
        elif name == "tnn":
            mt.mtnn_tnn(dA, dB, out.view, ws)
        else:
            label = mt.mtnn_auto(dA, dB, out.view, ws)
            assert label == mt.mtnn_select(m, n, k)
        sync()
        got, intact = out.host()
        assert intact
        check_gemm(pick(got), C, S, k, f"{name} {m}x{n}x{k}")
        outs[name] = got
    # rerun bit-identity (no atomics, fixed summation order)
    again = Guarded(m, n)
    mt.mtnn_nt(dA, dB, again.view)
    sync()
    assert again.host()[0].tobytes() == outs["nt"].tobytes()
    # the transposed B in the workspace is bit-exact
    bt = ws[: n * k * 4].view(torch.float32).view(k, n).cpu().numpy()
    assert bt.tobytes() == np.ascontiguousarray(B.T).tobytes()
    # the two alternatives agree with each other within twice the tolerance
    d = np.abs(pick(outs["nt"]).astype(np.float64) - pick(outs["tnn"]).astype(np.float64))
    assert (d / np.where(S > 0, S, 1)).max() <= 2e-5 * np.sqrt(k)


def test_config1_single_nt_256():
    check_all_paths(256, 256, 256, 1702, "uniform")


@pytest.mark.parametrize("shape,seed", zip(I.CONFIG2["shapes"], I.CONFIG2["seeds"]))
def test_config2_fc_layer_shapes(shape, seed):
    check_all_paths(*shape, seed, "uniform")


@pytest.mark.parametrize("shape,seed", zip(I.CONFIG4["shapes"], I.CONFIG4["seeds"]))
def test_config4_skinny_and_irregular(shape, seed):
    check_all_paths(*shape, seed, "normal")


@pytest.mark.parametrize("shape,seed", zip(I.CONFIG4["shapes"], I.CONFIG4["seeds"]))
def test_config4_full_size_with_leading_dimensions_padded_by_three(shape, seed):
    """The skinny and irregular shapes once more with every leading dimension = width + 3 (rows no longer
    16-byte aligned: the guarded kernels), NaN in the operands' padding and canaries around and inside C."""
    import torch
    m, n, k = shape
    A, B = I.nt_operands(m, n, k, seed, "normal")
    C, S = oracle.nt_ref(A, B, with_bound=True)
    dA, dB = dev_matrix(A, k + 3), dev_matrix(B, k + 3)
    ws = torch.empty(mt.mtnn_tnn_workspace_bytes(n, k), dtype=torch.uint8, device="cuda")
    results = {}
    for name in ("nt", "tnn", "auto"):
        out = Guarded(m, n, n + 3)
        if name == "nt":
            mt.mtnn_nt(dA, dB, out.view)
        elif name == "tnn":
            mt.mtnn_tnn(dA, dB, out.view, ws)
        else:
            assert mt.mtnn_auto(dA, dB, out.view, ws) == mt.mtnn_select(m, n, k)
        sync()
        got, intact = out.host()
        assert intact, f"{name}: wrote into the padding of C or outside it"
        check_gemm(got, C, S, k, f"{name} ld+3 {m}x{n}x{k}")
        results[name] = got
    bt = ws[: n * k * 4].view(torch.float32).view(k, n).cpu().numpy()
    assert bt.tobytes() == np.ascontiguousarray(B.T).tobytes()
    # NN alone on a padded B^T as well (ldb = n + 3)
    Bt = np.ascontiguousarray(B.T)
    out = Guarded(m, n, n + 3)
    mt.mtnn_nn(dA, dev_matrix(Bt, n + 3), out.view)
    sync()
    got, intact = out.host()
    assert intact
    check_gemm(got, C, S, k, f"nn ld+3 {m}x{n}x{k}")


def test_auto_without_workspace_runs_nt():
    A, B = I.nt_operands(128, 128, 128, 9)
    dA, dB = dev_matrix(A), dev_matrix(B)
    out = Guarded(128, 128)
    assert mt.mtnn_auto(dA, dB, out.view, None) == 1
    sync()
    C, S = oracle.nt_ref(A, B, with_bound=True)
    check_gemm(out.host()[0], C, S, 128)


@pytest.mark.parametrize("m,n,k", [(8192, 8192, 8192), (64, 8192, 8192), (8192, 64, 64), (2048, 8192, 512)])
def test_config3_sweep_corners_sampled_rows(m, n, k):
    # the largest sweep shapes: the oracle checks the first/last rows of tile boundaries plus a
    # pseudo-random sample of rows, every column
    seed = 10000
    rows = sorted(set([0, 1, m - 2, m - 1] + [r for r in (255, 256, 257, 4095, 4096) if r < m] +
                      [int(x) for x in I.uniform_ints(seed, 9, 24, 0, m - 1)]))
    check_all_paths(m, n, k, seed, "uniform", rows=np.array(rows))


def test_split_k_on_two_streams_uses_separate_scratch():
    """Split-k partial products live in a scratch buffer per stream: launches interleaved on two
    streams must not disturb each other."""
    import torch
    m, n, k = 96, 200, 4096
    A1, B1 = operands(mt.OP_NT, m, n, k, 700, dist="normal")
    A2, B2 = operands(mt.OP_NT, m, n, k, 701, dist="normal")
    C1, S1 = reference(mt.OP_NT, A1, B1)
    C2, S2 = reference(mt.OP_NT, A2, B2)
    d = [dev_matrix(x) for x in (A1, B1, A2, B2)]
    o1 = torch.empty((m, n), device="cuda")
    o2 = torch.empty((m, n), device="cuda")
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(20):
        mt.mtnn_gemm_ex(mt.OP_NT, 3, d[0], d[1], o1, stream=s1, splits=8)
        mt.mtnn_gemm_ex(mt.OP_NT, 3, d[2], d[3], o2, stream=s2, splits=8)
    torch.cuda.synchronize()
    check_gemm(o1.cpu().numpy(), C1, S1, k, "stream 1")
    check_gemm(o2.cpu().numpy(), C2, S2, k, "stream 2")


@pytest.mark.parametrize("which", ["A_rows", "B_rows", "C_elems"])
def test_offsets_beyond_2_to_31_elements(which):
    """Row offsets (row x ld) past 2^31 elements in A, in B and in C: 64-bit index arithmetic.
    Operands are drawn on the device by torch's seeded generator (not by this library) and only the
    sampled rows travel to the host for the oracle."""
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(31337)
    if which == "A_rows":
        m, n, k = 36000, 128, 65536          # A: 2.36e9 elements
    elif which == "B_rows":
        m, n, k = 128, 36000, 65536          # B: 2.36e9 elements
    else:
        m, n, k = 48000, 48000, 64           # C: 2.30e9 elements
    A = torch.rand((m, k), generator=gen, device="cuda").mul_(2).sub_(1)
    B = torch.rand((n, k), generator=gen, device="cuda").mul_(2).sub_(1)
    C = torch.full((m, n), float("nan"), device="cuda")
    ws = torch.empty(mt.mtnn_tnn_workspace_bytes(n, k), dtype=torch.uint8, device="cuda")
    rows = sorted({0, 1, m - 1, m - 2, m // 2, 32768 if m > 32768 else 5, 32769 if m > 32769 else 6, 35999 if m > 35999 else 7})
    cols = sorted({0, 1, n - 1, n - 2, n // 2, 32768 if n > 32768 else 5, 35999 if n > 35999 else 7})
    hA = A[rows].cpu().numpy()
    hB = B[cols].cpu().numpy()
    Cref, Sref = oracle.nt_ref(hA, hB, with_bound=True)
    for name in ("nt", "tnn"):
        C.fill_(float("nan"))
        if name == "nt":
            mt.mtnn_nt(A, B, C)
        else:
            mt.mtnn_tnn(A, B, C, ws)
        sync()
        got = C[rows][:, cols].cpu().numpy()
        check_gemm(got, Cref, Sref, k, f"{which} {name}")
    # spot-check that the far corner of the transposed B in the workspace is right
    bt = ws[: n * k * 4].view(torch.float32).view(k, n)
    assert torch.equal(bt[k - 1, n - 3:], B[n - 3:, k - 1])
    assert torch.equal(bt[:4, n - 1], B[n - 1, :4])
    del A, B, C, ws
    torch.cuda.empty_cache()


def _strided_on_device(x, ld):
    """rows x cols device view with leading dimension ld; the padding is left uninitialised."""
    import torch
    rows, cols = x.shape
    buf = torch.empty(rows * ld, dtype=torch.float32, device="cuda")
    view = buf.view(rows, ld)[:, :cols]
    view.copy_(torch.from_numpy(x).cuda())
    return view


@pytest.mark.parametrize("case", ["nt_A_guarded", "nt_A_pipelined", "nt_B_guarded", "nn_B_guarded", "nn_B_pipelined"])
def test_huge_leading_dimensions(case):
    """Leading dimensions so large that byte offsets inside one tile reach 2^32: the pipelined kernel
    addresses a tile with 32-bit lane offsets, so such calls must take the guarded kernel; a leading
    dimension just under the limit stays on the pipelined kernel with offsets close to 2^32."""
    import torch
    if case.startswith("nt"):
        op, m, n, k = mt.OP_NT, 70, 72, 96
        A, B = operands(op, m, n, k, 8800)
        big = (1 << 22) + 4
        if case == "nt_A_guarded":        # 256 rows x lda x 4 B >= 2^32
            cfg, dA, dB = 0, _strided_on_device(A, big), _strided_on_device(B, k)
        elif case == "nt_A_pipelined":    # 64 rows x lda x 4 B just above 2^30
            cfg, dA, dB = 3, _strided_on_device(A, big), _strided_on_device(B, k)
        else:
            cfg, dA, dB = 0, _strided_on_device(A, k), _strided_on_device(B, big)
    else:
        op, m, n, k = mt.OP_NN, 70, 72, 40
        A, B = operands(op, m, n, k, 8801)
        ldb = (1 << 26) if case == "nn_B_guarded" else (1 << 24)      # (BK + 1) x ldb x 4 B vs 2^32
        cfg, dA, dB = 0, _strided_on_device(A, k), _strided_on_device(B, ldb)
    out = Guarded(m, n, n + 4)
    mt.mtnn_gemm_ex(op, cfg, dA, dB, out.view)
    sync()
    got, intact = out.host()
    assert intact
    Cref, Sref = reference(op, A, B)
    check_gemm(got, Cref, Sref, k, case)
    del dA, dB
    torch.cuda.empty_cache()


@pytest.mark.parametrize("op", [mt.OP_NT, mt.OP_NN], ids=["NT", "NN"])
@pytest.mark.parametrize("cfg", [10, 11, 12, 13, 14, 15])
def test_several_workgroups_per_cu_on_a_full_grid(op, cfg):
    """Configurations that put two or three workgroups on a CU, on a grid large enough that every CU
    really holds that many (768+ tiles), with a ragged last slab."""
    m, n, k = 3072, 2048, 72
    A, B = operands(op, m, n, k, 900 + cfg)
    got = run(op, cfg, A, B)
    C, S = reference(op, A, B)
    check_gemm(got, C, S, k, f"op{op} cfg{cfg}")


@pytest.mark.parametrize("op", [mt.OP_NT, mt.OP_NN], ids=["NT", "NN"])
@pytest.mark.parametrize("cfg", [3, 6, 8, 9, 10, 11, 12, 13, 14, 15])
def test_even_cut_against_oracle(op, cfg):
    """splits = EVEN_CUT: all tiles' k ranges cut into equal pieces over a fixed grid, cut tiles
    finished by the fix-up kernel; ragged m, n edges and a ragged last k unit."""
    m, n, k = 1000, 900, 1100
    A, B = operands(op, m, n, k, 950 + cfg, dist="normal")
    before = mt.mtnn_gemm_even_cut_launches()
    got = run(op, cfg, A, B, ldc=n + 4, splits=mt.EVEN_CUT)
    assert mt.mtnn_gemm_even_cut_launches() == before + 1, "the launch did not take the even-cut path"
    C, S = reference(op, A, B)
    check_gemm(got, C, S, k, f"op{op} cfg{cfg} even cut")
    again = run(op, cfg, A, B, ldc=n + 4, splits=mt.EVEN_CUT)
    assert again.tobytes() == got.tobytes()            # fixed cut, fixed order of the pieces


def test_even_cut_integer_inputs_bit_exact_and_fallback():
    for op in (mt.OP_NT, mt.OP_NN):
        A, B = operands(op, 1500, 700, 2048, 960, dist="int")
        C, _ = reference(op, A, B)
        before = mt.mtnn_gemm_even_cut_launches()
        got = run(op, 10, A, B, splits=mt.EVEN_CUT)
        assert mt.mtnn_gemm_even_cut_launches() == before + 1
        assert np.array_equal(got, C.astype(np.float32))
        # fewer units than pieces, or operands the pipelined kernel cannot take: runs unsplit, still right
        A2, B2 = operands(op, 130, 132, 64, 961, dist="int")
        C2, _ = reference(op, A2, B2)
        assert np.array_equal(run(op, 10, A2, B2, splits=mt.EVEN_CUT), C2.astype(np.float32))
        A3, B3 = operands(op, 1000, 900, 1101, 962, dist="int")          # k % 4 != 0
        C3, _ = reference(op, A3, B3)
        assert np.array_equal(run(op, 10, A3, B3, splits=mt.EVEN_CUT), C3.astype(np.float32))
