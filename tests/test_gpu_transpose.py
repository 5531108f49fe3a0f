"""mtnn_transpose against the CPU oracle: bit-exact, including padding and guard bands."""
import numpy as np
import pytest

import oracle
from paper_1702_03192_amd import binding as mt
from paper_1702_03192_amd import inputs as I
from gpu_util import CANARY_BITS, Guarded, check_gemm, dev_matrix

pytestmark = pytest.mark.gpu


def run_transpose(x, ldin=None, ldout=None, misalign=0):
    import torch
    rows, cols = x.shape
    d_in = dev_matrix(x, ldin, misalign=misalign)
    out = Guarded(cols, rows, ldout, misalign=misalign)
    mt.mtnn_transpose(d_in, out.view)
    torch.cuda.synchronize()
    got, intact = out.host()
    assert intact, "transpose wrote outside its logical output"
    return got


@pytest.mark.parametrize("rows,cols", [(64, 64), (128, 192), (5, 7), (1, 300), (300, 1), (65, 63), (257, 130),
                                       (1000, 10), (10, 1000), (4500, 1500), (4096, 1024), (1024, 4096)])
def test_transpose_bit_exact(rows, cols):
    x = I.uniform_pm1(6000, 0, rows, cols)
    got = run_transpose(x)
    want = np.ascontiguousarray(oracle.transpose_ref(x))
    assert got.tobytes() == want.tobytes()


def test_transpose_index_coded_4096():
    x = I.index_coded(4096, 4096)
    got = run_transpose(x)
    assert got.tobytes() == np.ascontiguousarray(oracle.transpose_ref(x)).tobytes()


@pytest.mark.parametrize("rows,cols,ldin,ldout,mis", [(130, 70, 73, 133, 0), (128, 128, 132, 136, 0),
                                                      (128, 128, 128, 128, 1), (64, 200, 200, 67, 3),
                                                      (200, 64, 64, 200, 2)])
def test_transpose_leading_dims_padding_and_alignment(rows, cols, ldin, ldout, mis):
    x = I.normal01(6001, 0, rows, cols)
    got = run_transpose(x, ldin, ldout, misalign=mis)
    assert got.tobytes() == np.ascontiguousarray(oracle.transpose_ref(x)).tobytes()


def test_transpose_preserves_nan_payloads_and_signed_zero():
    rng_bits = (I._bits(6002, 0, 96, 160) >> np.uint64(32)).astype(np.uint32)   # arbitrary 32-bit patterns
    rng_bits[0, 0] = 0x7FC00001
    rng_bits[1, 2] = 0x80000000
    rng_bits[95, 159] = 0xFFC12345
    x = rng_bits.view(np.float32)
    got = run_transpose(x)
    assert np.array_equal(got.view(np.uint32), rng_bits.T)


def test_transpose_large_sampled_full_size():
    # 8192 x 8192 (the largest B of the sweep): whole-matrix comparison against the oracle
    x = I.uniform_pm1(6003, 0, 8192, 8192)
    got = run_transpose(x)
    want = np.ascontiguousarray(oracle.transpose_ref(x))
    assert got.tobytes() == want.tobytes()


@pytest.mark.parametrize("rows,cols,pad", [(4100, 4204, 0), (4100, 4204, 4),      # 128 x 64 tiles, ragged edges
                                           (8196, 8260, 0), (8196, 8260, 8),      # 256 x 64 tiles, ragged edges
                                           (300, 70000, 0), (70000, 300, 4),      # long and thin
                                           (8195, 8201, 0)])                      # large and not 16-byte friendly
def test_transpose_large_tile_shapes_with_edges(rows, cols, pad):
    """The tile shapes used for matrices beyond 2^24 and 2^26 elements, with partial edge tiles and padded rows."""
    x = I.uniform_pm1(6005, 0, rows, cols)
    got = run_transpose(x, cols + pad, rows + 2 * pad)
    assert got.tobytes() == np.ascontiguousarray(oracle.transpose_ref(x)).tobytes()


def test_transpose_empty_is_a_noop():
    import torch
    out = Guarded(0, 5)
    x = torch.empty((5, 0), dtype=torch.float32, device="cuda")
    assert mt.lib().mtnn_transpose(None, 5, 0, x.data_ptr(), 1, out.view.data_ptr(), 5) == 0
    assert mt.lib().mtnn_transpose(None, 0, 5, x.data_ptr(), 5, out.view.data_ptr(), 1) == 0
    torch.cuda.synchronize()
    assert out.host()[1]


def test_transpose_involution_on_device():
    import torch
    x = I.normal01(6004, 0, 777, 333)
    d = dev_matrix(x)
    t1 = torch.empty((333, 777), dtype=torch.float32, device="cuda")
    t2 = torch.empty((777, 333), dtype=torch.float32, device="cuda")
    mt.mtnn_transpose(d, t1)
    mt.mtnn_transpose(t1, t2)
    torch.cuda.synchronize()
    assert t2.cpu().numpy().tobytes() == x.tobytes()


@pytest.mark.parametrize("n,ld", [(64, 64), (1, 1), (5, 9), (130, 130), (257, 300), (1000, 1000), (4096, 4096),
                                  (72, 76), (4100, 4104), (8192, 8192)])
def test_inplace_square_transpose_bit_exact(n, ld):
    import torch
    x = I.normal01(6100, 0, n, n)
    d = dev_matrix(x, ld, fill=np.float32(-3.0))
    base = d.storage_offset()
    mt.mtnn_transpose_inplace(d)
    torch.cuda.synchronize()
    assert d.cpu().numpy().tobytes() == np.ascontiguousarray(oracle.transpose_ref(x)).tobytes()
    if ld > n:                                           # padding untouched
        full = d.as_strided((n, ld), (ld, 1), base).cpu().numpy()
        assert np.all(full[:, n:] == -3.0)
    mt.mtnn_transpose_inplace(d)
    torch.cuda.synchronize()
    assert d.cpu().numpy().tobytes() == x.tobytes()


def test_tnn_inplace_matches_oracle_and_restores_b():
    import torch
    from gpu_util import check_gemm
    m, n = 300, 520
    A, B = I.nt_operands(m, n, n, 6200, "normal")
    dA, dB = dev_matrix(A), dev_matrix(B)
    out = Guarded(m, n)
    mt.mtnn_tnn_inplace(dA, dB, out.view)
    torch.cuda.synchronize()
    got, intact = out.host()
    assert intact
    C, S = oracle.nt_ref(A, B, with_bound=True)
    check_gemm(got, C, S, n, "tnn_inplace")
    assert dB.cpu().numpy().tobytes() == B.tobytes()
    with pytest.raises(mt.MtnnError) as e:          # a rectangular B must be dense
        mt.mtnn_tnn_inplace(dA[:, :100].contiguous(), dev_matrix(B[:, :100].copy(), 104), out.view)
    assert e.value.status == 8


# ---- rectangular in-place transposition -------------------------------------------------------------

RECT_SHAPES = [(2, 3), (3, 2), (5, 7), (97, 3), (3, 97), (31, 17), (127, 251), (251, 127), (1009, 13),   # prime dimensions
               (24, 36), (36, 24), (64, 48), (100, 1000), (1000, 100), (96, 4096), (4096, 96),            # a common factor: three passes
               (1, 9), (9, 1), (1024, 2048), (2048, 1024), (1500, 4500), (4097, 1023), (33, 32768), (32768, 33),
               (8192, 4096), (300, 301)]


@pytest.mark.parametrize("rows,cols", RECT_SHAPES, ids=lambda v: str(v))
def test_rectangular_inplace_transpose_is_bit_exact_and_its_own_inverse(rows, cols):
    """rows x cols dense -> cols x rows dense in the same buffer, against the oracle's transpose word for
    word (an index-coded matrix, so a misplaced word shows), canaries on both sides, and back again."""
    import torch
    guard = 64
    if rows * cols < (1 << 24):        # every word distinct and exact in fp32: word e holds the value e
        x = np.arange(rows * cols, dtype=np.float32).reshape(rows, cols)
    else:
        x = I.uniform_pm1(77, 0, rows, cols)
    host = np.full(guard + rows * cols + guard, np.float32(np.nan), dtype=np.float32)
    host[:guard].view(np.uint32)[:] = 0x7FC0DEAD
    host[guard + rows * cols:].view(np.uint32)[:] = 0x7FC0DEAD
    host[guard:guard + rows * cols] = x.reshape(-1)
    buf = torch.from_numpy(host).cuda()
    body = buf[guard:guard + rows * cols]
    mt.mtnn_transpose_inplace_rect(body, rows, cols)
    torch.cuda.synchronize()
    got = buf.cpu().numpy()
    want = np.ascontiguousarray(oracle.transpose_ref(x)).reshape(-1)
    assert got[guard:guard + rows * cols].tobytes() == want.tobytes()
    assert (got[:guard].view(np.uint32) == 0x7FC0DEAD).all() and (got[guard + rows * cols:].view(np.uint32) == 0x7FC0DEAD).all()
    mt.mtnn_transpose_inplace_rect(body, cols, rows)
    torch.cuda.synchronize()
    assert buf.cpu().numpy()[guard:guard + rows * cols].tobytes() == x.reshape(-1).tobytes()


def test_rectangular_inplace_transpose_keeps_nan_payloads_and_signed_zeros():
    import torch
    rows, cols = 37, 52
    bits = I.uniform_ints(99, 0, rows * cols, 0, 2 ** 31 - 1).astype(np.uint32) * np.uint32(2) + np.uint32(1)
    bits[:4] = [0x80000000, 0x7FC00001, 0xFFC12345, 0x00000001]
    buf = torch.from_numpy(bits.view(np.float32).copy()).cuda()
    mt.mtnn_transpose_inplace_rect(buf, rows, cols)
    torch.cuda.synchronize()
    assert buf.cpu().numpy().view(np.uint32).tobytes() == np.ascontiguousarray(bits.reshape(rows, cols).T).tobytes()


@pytest.mark.parametrize("m,n,k", [(100, 96, 260), (257, 1000, 100), (64, 127, 251), (300, 2048, 1024)])
def test_tnn_through_rectangular_inplace_transposes_matches_oracle_and_restores_b(m, n, k):
    import torch
    A, B = I.nt_operands(m, n, k, 4400 + n, "normal")
    C, S = oracle.nt_ref(A, B, with_bound=True)
    dA, dB = dev_matrix(A), dev_matrix(B)
    out = Guarded(m, n, n + 4)
    mt.mtnn_tnn_inplace(dA, dB, out.view)
    torch.cuda.synchronize()
    got, intact = out.host()
    assert intact
    check_gemm(got, C, S, k, f"in-place TNN {m}x{n}x{k}")
    assert dB.cpu().numpy().tobytes() == B.tobytes(), "B was not restored"


def test_three_way_choice_runs_each_forced_path_and_the_rule():
    import torch
    m, n, k = 200, 328, 124
    A, B = I.nt_operands(m, n, k, 4500, "uniform")
    C, S = oracle.nt_ref(A, B, with_bound=True)
    dA, dB = dev_matrix(A), dev_matrix(B)
    ws = torch.full((mt.mtnn_tnn_workspace_bytes(n, k) // 4,), float("nan"), device="cuda")
    for mode, workspace in ((1, None), (-1, ws), (-2, None), (0, ws), (0, None)):
        out = Guarded(m, n)
        chosen = mt.mtnn_auto3(dA, dB, out.view, workspace, mode)
        torch.cuda.synchronize()
        got, intact = out.host()
        assert intact
        check_gemm(got, C, S, k, f"auto3 mode {mode} -> {chosen}")
        if mode != 0:
            assert chosen == mode
        else:
            assert chosen == mt.mtnn_select3(m, n, k, workspace is not None, True)
        assert dB.cpu().numpy().tobytes() == B.tobytes()
    bt = ws[: n * k].view(k, n).cpu().numpy()
    assert bt.tobytes() == np.ascontiguousarray(B.T).tobytes()          # the forced TNN went through the workspace
    with pytest.raises(mt.MtnnError) as e:
        mt.mtnn_auto3(dA, dB, Guarded(m, n).view, None, -1)
    assert e.value.status == 5
