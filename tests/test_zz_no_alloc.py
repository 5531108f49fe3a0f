"""mtnn_gemm_ex_static (the entry point that allocates nothing: partial products of divided launches in
the library's own static device array) against mtnn_gemm_ex with lent scratch: same kernels, same
division, so the same bits; plus the fp64 oracle, the size limit, and a smaller call after a larger
one on the shared array."""
import numpy as np
import pytest

import oracle
from paper_1702_03192_amd import binding as mt
from paper_1702_03192_amd import inputs as I
from gpu_util import Guarded, check_gemm, dev_matrix

pytestmark = pytest.mark.gpu

STATIC_BYTES = 32 << 20


def _both(op, cfg, splits, m, n, k, seed):
    """The static entry point and the ordinary one on the same operands; returns the static result after
    checking it against the ordinary one bit for bit and against the oracle."""
    import torch
    A, B = I.nt_operands(m, n, k, seed, "normal")
    if op == mt.OP_NN:
        B = np.ascontiguousarray(B.T)
    C, S = (oracle.nt_ref if op == mt.OP_NT else oracle.nn_ref)(A, B, with_bound=True)
    dA, dB = dev_matrix(A), dev_matrix(B)
    want = Guarded(m, n, n + 4)
    mt.mtnn_gemm_ex(op, cfg, dA, dB, want.view, splits=splits)
    got = Guarded(m, n, n + 4)
    mt.mtnn_gemm_ex_static(op, cfg, dA, dB, got.view, splits=splits)
    torch.cuda.synchronize()
    w, w_ok = want.host()
    g, g_ok = got.host()
    assert w_ok and g_ok
    check_gemm(g, C, S, k, f"static op{op} cfg{cfg} splits{splits} {m}x{n}x{k}")
    assert g.tobytes() == w.tobytes(), "static and lent scratch must give the same bits"
    return g


@pytest.mark.parametrize("op", [mt.OP_NT, mt.OP_NN], ids=["NT", "NN"])
def test_two_calls_in_a_row_the_second_smaller(op):
    first = _both(op, 3, 8, 300, 264, 2052, 9100)            # split-k: 8 partial products of 300 x 264
    second = _both(op, 3, 4, 70, 92, 1000, 9101)             # a smaller product over the same array
    assert first.shape == (300, 264) and second.shape == (70, 92)
    # the first call again: what the second left in the array does not matter
    again = _both(op, 3, 8, 300, 264, 2052, 9100)
    assert again.tobytes() == first.tobytes()


@pytest.mark.parametrize("op", [mt.OP_NT, mt.OP_NN], ids=["NT", "NN"])
def test_even_cut_and_the_rules_own_choice(op):
    before = mt.mtnn_gemm_even_cut_launches()
    _both(op, 9, mt.EVEN_CUT, 1000, 900, 1100, 9200)         # 64 x 128 tiles: 2 x 512 slots of 32 KB = 32 MiB exactly
    assert mt.mtnn_gemm_even_cut_launches() == before + 2
    _both(op, 9, mt.EVEN_CUT, 520, 380, 900, 9201)           # smaller, straight after
    # cfg = -1, splits = 0: the rule, told about 32 MiB; a shape it splits
    m, n, k = 64, 128, 8192
    cfg, splits = mt.mtnn_gemm_choice(op, m, n, k, STATIC_BYTES)
    assert splits > 1
    import torch
    A, B = I.nt_operands(m, n, k, 9202, "normal")
    if op == mt.OP_NN:
        B = np.ascontiguousarray(B.T)
    dA, dB = dev_matrix(A), dev_matrix(B)
    by_rule = torch.empty((m, n), device="cuda")
    by_name = torch.empty((m, n), device="cuda")
    mt.mtnn_gemm_ex_static(op, -1, dA, dB, by_rule)
    mt.mtnn_gemm_ex_static(op, cfg, dA, dB, by_name, splits=splits)
    torch.cuda.synchronize()
    assert by_rule.cpu().numpy().tobytes() == by_name.cpu().numpy().tobytes()
    C, S = (oracle.nt_ref if op == mt.OP_NT else oracle.nn_ref)(A, B, with_bound=True)
    check_gemm(by_rule.cpu().numpy(), C, S, k, "rule's choice")


def test_sizes_beyond_the_array_are_refused_and_nothing_is_written():
    import torch
    m, n, k = 2048, 2048, 512
    assert mt.mtnn_gemm_scratch_bytes(3, 4, m, n, k) == 4 * m * n * 4 > STATIC_BYTES
    A = torch.zeros((m, k), device="cuda")
    B = torch.zeros((n, k), device="cuda")
    out = torch.full((m, n), 7.0, device="cuda")
    with pytest.raises(mt.MtnnError) as e:
        mt.mtnn_gemm_ex_static(mt.OP_NT, 3, A, B, out, splits=4)
    assert e.value.status == 5
    with pytest.raises(mt.MtnnError) as e:                    # 128 x 128 tiles: the even cut's slots need 64 MiB
        mt.mtnn_gemm_ex_static(mt.OP_NT, 10, A, B, out, splits=mt.EVEN_CUT)
    assert e.value.status == 5
    torch.cuda.synchronize()
    assert float(out.min().item()) == 7.0 and float(out.max().item()) == 7.0
    # exactly at the limit is accepted: 2 partial products of 2048 x 2048
    assert mt.mtnn_gemm_scratch_bytes(3, 2, m, n, k) == STATIC_BYTES
    mt.mtnn_gemm_ex_static(mt.OP_NT, 3, A, B, out, splits=2)
    torch.cuda.synchronize()
    assert float(out.abs().max().item()) == 0.0
    # the registered scratch plays no part: withdraw it from the stream and the static call still splits
    s = torch.cuda.Stream()
    mt.lend_scratch(s, 0)
    mt.mtnn_gemm_ex_static(mt.OP_NT, 3, A, B, out, stream=s, splits=2)
    s.synchronize()
    mt.lend_scratch(s)
