"""Scratch memory for divided launches is the caller's: the library allocates nothing, divides a
product the same way whenever the same capacity is registered for the stream (eager or under
capture), refuses an explicit division that does not fit, and runs unsplit when nothing is lent."""
import numpy as np
import pytest

import oracle
from paper_1702_03192_amd import binding as mt
from paper_1702_03192_amd import inputs as I
from gpu_util import check_gemm, dev_matrix

pytestmark = pytest.mark.gpu


def _operands(m, n, k, seed):
    A, B = I.nt_operands(m, n, k, seed, "normal")
    return A, B, dev_matrix(A), dev_matrix(B)


def test_explicit_split_needs_scratch_and_auto_runs_unsplit_without_it():
    import torch
    m, n, k = 96, 200, 4096
    A, B, dA, dB = _operands(m, n, k, 7100)
    C, S = oracle.nt_ref(A, B, with_bound=True)
    s = torch.cuda.Stream()
    out = torch.empty((m, n), device="cuda")
    try:
        mt.lend_scratch(s, 0)                                   # nothing lent on this stream
        assert mt.mtnn_get_scratch_bytes(s) == 0
        with pytest.raises(mt.MtnnError) as e:
            mt.mtnn_gemm_ex(mt.OP_NT, 3, dA, dB, out, stream=s, splits=8)
        assert e.value.status == 5
        with pytest.raises(mt.MtnnError) as e:
            mt.mtnn_gemm_ex(mt.OP_NT, 3, dA, dB, out, stream=s, splits=2)
        assert e.value.status == 5
        # the rule's own choice with no scratch is an unsplit launch, bit-identical to that launch asked for by name
        cfg0, splits0 = mt.mtnn_gemm_choice(mt.OP_NT, m, n, k, 0)
        assert splits0 == 1
        mt.mtnn_nt(dA, dB, out, stream=s)
        s.synchronize()
        got = out.cpu().numpy()
        check_gemm(got, C, S, k, "no scratch")
        by_name = torch.empty_like(out)
        mt.mtnn_gemm_ex(mt.OP_NT, cfg0, dA, dB, by_name, stream=s, splits=1)
        s.synchronize()
        assert by_name.cpu().numpy().tobytes() == got.tobytes()
        # a small loan: only divisions that fit it are considered, and an explicit one beyond it is refused
        need4 = mt.mtnn_gemm_scratch_bytes(3, 4, m, n, k)
        mt.lend_scratch(s, need4)
        assert mt.mtnn_get_scratch_bytes(s) == need4
        mt.mtnn_gemm_ex(mt.OP_NT, 3, dA, dB, out, stream=s, splits=4)
        s.synchronize()
        check_gemm(out.cpu().numpy(), C, S, k, "splits 4 in an exact loan")
        with pytest.raises(mt.MtnnError) as e:
            mt.mtnn_gemm_ex(mt.OP_NT, 3, dA, dB, out, stream=s, splits=8)
        assert e.value.status == 5
        cfg1, splits1 = mt.mtnn_gemm_choice(mt.OP_NT, m, n, k, need4)
        assert splits1 in (1, 2, 4)
        mt.mtnn_nt(dA, dB, out, stream=s)
        s.synchronize()
        got1 = out.cpu().numpy()
        mt.mtnn_gemm_ex(mt.OP_NT, cfg1, dA, dB, by_name, stream=s, splits=splits1)
        s.synchronize()
        assert by_name.cpu().numpy().tobytes() == got1.tobytes()
    finally:
        mt.lend_scratch(s)                                      # back to the default capacity


@pytest.mark.parametrize("op", [mt.OP_NT, mt.OP_NN], ids=["NT", "NN"])
def test_a_split_launch_gives_the_same_bits_eagerly_and_from_a_graph(op):
    """The default rule splits k for this shape; the same call captured into a graph (scratch lent to
    the stream beforehand) must give the eager call's bits on every replay, with eager work between."""
    import torch
    m, n, k = 64, 128, 8192
    A, B = I.nt_operands(m, n, k, 7200, "normal")
    if op == mt.OP_NN:
        B = np.ascontiguousarray(B.T)
    ref = (oracle.nt_ref if op == mt.OP_NT else oracle.nn_ref)(A, B, with_bound=True)
    dA, dB = dev_matrix(A), dev_matrix(B)
    cfg, splits = mt.mtnn_gemm_choice(op, m, n, k)
    assert splits > 1, "this shape is meant to be one the rule splits"
    s = torch.cuda.Stream()
    fn = mt.mtnn_nt if op == mt.OP_NT else mt.mtnn_nn
    mt.lend_scratch(s)
    eager = torch.empty((m, n), device="cuda")
    fn(dA, dB, eager, stream=s)
    s.synchronize()
    want = eager.cpu().numpy()
    check_gemm(want, ref[0], ref[1], k, "eager")
    captured = torch.full((m, n), float("nan"), device="cuda")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        fn(dA, dB, captured)
    other = torch.zeros(1 << 18, device="cuda")
    for i in range(4):
        captured.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert captured.cpu().numpy().tobytes() == want.tobytes(), f"replay {i}"
        other.add_(1.0)
        assert float(other.sum().item()) == (i + 1) * (1 << 18)
    # ... and the same once more eagerly on another stream with its own loan of the same size
    s2 = torch.cuda.Stream()
    again = torch.empty((m, n), device="cuda")
    fn(dA, dB, again, stream=s2)
    s2.synchronize()
    assert again.cpu().numpy().tobytes() == want.tobytes()
