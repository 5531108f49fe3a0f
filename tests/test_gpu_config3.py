"""Every one of the 512 shapes of the sweep grid {64, ..., 8192}^3 against the fp64 oracle: the direct
NT kernel, TNN and the selected path, each with the configuration, split count and division the
library's own rule picks for that shape.

Operands: uniform [-1, 1) drawn on the device by torch's seeded generator (seed 10000 + 64 i_m + 8 i_n
+ i_k, the sweep's recipe) and copied to the host for the oracle.  Shapes of at most 2^36
multiply-adds are checked in full; above that, the first and last two rows of every 256-row block plus
64 seeded rows, all n columns.  Element-wise, both readings of 1e-5 sqrt(k)."""
import numpy as np
import pytest

import oracle
from paper_1702_03192_amd import binding as mt
from paper_1702_03192_amd import inputs as I
from gpu_util import check_gemm, check_gemm_on_device

pytestmark = pytest.mark.gpu

SIZES = (64, 128, 256, 512, 1024, 2048, 4096, 8192)
FULL_LIMIT = 1 << 36
SHAPES = [(im, inn, ik) for im in range(8) for inn in range(8) for ik in range(8)]


def sample_rows(m, seed):
    rows = set()
    for b in range(0, m, 256):
        rows.update((b, b + 1, min(b + 254, m - 1), min(b + 255, m - 1)))
    rows.update(int(x) for x in I.uniform_ints(seed, 9, 64, 0, m - 1))
    return np.array(sorted(rows))


@pytest.mark.parametrize("im,inn,ik", SHAPES, ids=[f"{SIZES[a]}x{SIZES[b]}x{SIZES[c]}" for a, b, c in SHAPES])
def test_sweep_shape_all_paths(im, inn, ik):
    import torch
    m, n, k = SIZES[im], SIZES[inn], SIZES[ik]
    seed = 10000 + 64 * im + 8 * inn + ik
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    A = torch.rand((m, k), generator=gen, device="cuda").mul_(2).sub_(1)
    B = torch.rand((n, k), generator=gen, device="cuda").mul_(2).sub_(1)
    ws = torch.empty(mt.mtnn_tnn_workspace_bytes(n, k), dtype=torch.uint8, device="cuda")
    C_nt = torch.full((m, n), float("nan"), device="cuda")
    C_tnn = torch.full((m, n), float("nan"), device="cuda")
    C_auto = torch.full((m, n), float("nan"), device="cuda")
    mt.mtnn_nt(A, B, C_nt)
    mt.mtnn_tnn(A, B, C_tnn, ws)
    label = mt.mtnn_auto(A, B, C_auto, ws)
    torch.cuda.synchronize()
    # Algorithm 2 ran the path the predictor names, and its result is that path's, bit for bit
    assert label == mt.mtnn_select(m, n, k) and label in (1, -1)
    assert torch.equal(C_auto, C_nt if label == 1 else C_tnn)
    # Algorithm 1 left B^T in the workspace, bit-exact
    bt = ws[: n * k * 4].view(torch.float32).view(k, n)
    assert torch.equal(bt, B.t())
    hA, hB = A.cpu().numpy(), B.cpu().numpy()
    rows = None if m * n * k <= FULL_LIMIT else sample_rows(m, seed)
    C, S = oracle.nt_ref(hA, hB, rows=rows, with_bound=True)
    for name, out in (("nt", C_nt), ("tnn", C_tnn)):
        got = out if rows is None else out[torch.from_numpy(rows).cuda()]
        what = f"{name} {m}x{n}x{k}"
        if got.numel() <= (1 << 20):
            check_gemm(got.cpu().numpy(), C, S, k, what)
        else:
            check_gemm_on_device(got, C, S, k, what)
    del A, B, ws, C_nt, C_tnn, C_auto


def test_the_grid_exercises_many_configurations_and_divisions():
    """The point of checking every shape: the rule picks different (configuration, division) pairs over
    the grid, for NT and for NN (the second half of TNN), and all of them went through the test above."""
    picks = {op: set() for op in (mt.OP_NT, mt.OP_NN)}
    for im, inn, ik in SHAPES:
        for op in picks:
            picks[op].add(mt.mtnn_gemm_choice(op, SIZES[im], SIZES[inn], SIZES[ik]))
    for op, seen in picks.items():
        assert len(seen) >= 9 and len({c for c, _ in seen}) >= 5, seen
        assert any(s > 1 for _, s in seen), seen             # split-k among them
