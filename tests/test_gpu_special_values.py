"""Non-finite and subnormal values through the GEMM kernels.

Eq. 1 / Eq. 2 are plain sums of products, so IEEE arithmetic fixes what an infinity or a NaN in an
operand does: it reaches exactly the results whose sum contains it (a row of C for an element of A, a
column for an element of B) and nothing else.  The kernels clamp out-of-range rows to valid ones,
zero-fill the k tail and, when the k range is divided, add partial products -- each a place where a
stray value could leak into, or vanish from, results it does not belong to.  The oracle evaluates
the same sums in double precision, where infinities and NaNs arise in exactly the same places (no
finite partial sum of these inputs overflows in either precision).
"""
import numpy as np
import pytest

import oracle
from paper_1702_03192_amd import binding as mt
from paper_1702_03192_amd import inputs as I
from gpu_util import tol
from test_gpu_gemm import operands, reference, run

pytestmark = pytest.mark.gpu

# (m, n, k, cfg, splits): the pipelined kernel on full and ragged tiles, the guarded kernel (k not a
# multiple of 4), the largest tile, a two-wave-set configuration, split-k, the even cut, the rule's choice
CASES = [(256, 384, 128, -1, 0), (300, 264, 200, 9, 0), (131, 262, 45, -1, 0), (257, 300, 72, 0, 0),
         (200, 136, 512, 13, 0), (70, 92, 1000, 3, 4), (300, 264, 2052, -1, 0), (1000, 900, 1100, 12, mt.EVEN_CUT)]


def plant(op, A, B):
    """Infinities and NaNs at fixed places: first / interior / last rows, first and last k."""
    m, k = A.shape
    A[3, 5 % k] = np.nan
    A[10, 0] = np.inf
    A[m - 1, k - 1] = -np.inf
    if op == mt.OP_NT:                 # B is n x k
        B[7, k - 1] = np.inf
        B[20, 2 % k] = np.nan
        B[B.shape[0] - 1, 0] = -np.inf
    else:                              # B is k x n
        B[k - 1, 7] = np.inf
        B[2 % k, 20] = np.nan
        B[0, B.shape[1] - 1] = -np.inf


@pytest.mark.parametrize("op", [mt.OP_NT, mt.OP_NN], ids=["NT", "NN"])
@pytest.mark.parametrize("m,n,k,cfg,splits", CASES, ids=[f"{c[0]}x{c[1]}x{c[2]}_cfg{c[3]}_s{c[4]}" for c in CASES])
def test_infinities_and_nans_reach_exactly_the_results_the_definition_says(op, m, n, k, cfg, splits):
    A, B = operands(op, m, n, k, 900 + k)
    plant(op, A, B)
    with np.errstate(invalid="ignore", over="ignore"):
        C, S = reference(op, A, B)
    got = run(op, cfg, A, B, splits=splits).astype(np.float64)
    nan_ref, inf_ref = np.isnan(C), np.isinf(C)
    # the planted values must have reached whole rows and columns, or the case tests nothing
    assert nan_ref[3].all() and nan_ref[:, 20].all() and inf_ref.any() and (~(nan_ref | inf_ref)).sum() > m * n // 2
    assert np.array_equal(np.isnan(got), nan_ref), "NaNs in other places than the definition's"
    assert np.array_equal(np.isinf(got), inf_ref), "infinities in other places than the definition's"
    assert np.array_equal(got[inf_ref], C[inf_ref]), "an infinity of the wrong sign"
    fin = ~(nan_ref | inf_ref)
    err = float((np.abs(got[fin] - C[fin]) / S[fin]).max())
    assert err <= tol(k), f"finite results next to non-finite ones: error {err:.3e} > {tol(k):.3e}"


def test_tnn_carries_non_finite_values_like_nt():
    """The transpose moves bit patterns, so TNN sees the same special values as NT."""
    import torch
    m, n, k = 200, 328, 124
    A, B = I.nt_operands(m, n, k, seed=977)
    plant(mt.OP_NT, A, B)
    with np.errstate(invalid="ignore", over="ignore"):
        C, S = oracle.nt_ref(A, B, with_bound=True)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    ws = torch.empty(mt.mtnn_tnn_workspace_bytes(n, k), dtype=torch.uint8, device="cuda")
    out = torch.empty((m, n), dtype=torch.float32, device="cuda")
    mt.mtnn_tnn(dA, dB, out, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(C)) and np.array_equal(np.isinf(got), np.isinf(C))
    fin = np.isfinite(C)
    assert np.array_equal(got[np.isinf(C)], C[np.isinf(C)])
    assert float((np.abs(got[fin] - C[fin]) / S[fin]).max()) <= tol(k)


# scale of A, scale of B: products that are subnormal, subnormal inputs, results around the smallest normal number
SUBNORMAL_CASES = [(2.0 ** -70, 2.0 ** -70), (2.0 ** -130, 8.0), (2.0 ** -64, 2.0 ** -62)]


@pytest.mark.parametrize("op", [mt.OP_NT, mt.OP_NN], ids=["NT", "NN"])
@pytest.mark.parametrize("sa,sb", SUBNORMAL_CASES, ids=["products", "inputs", "results"])
@pytest.mark.parametrize("m,n,k", [(128, 256, 64), (131, 262, 45), (70, 92, 1000)])
def test_subnormal_inputs_and_results_are_kept_not_flushed(op, sa, sb, m, n, k):
    """Gradual underflow: with operands scaled so that inputs, products or sums are subnormal in fp32, the
    result stays within the format's own limit of the exact sum -- half a unit of the subnormal spacing
    2^-149 per product (sums of subnormals are exact), on top of the usual relative tolerance where the
    sum is a normal number.  A kernel that flushed subnormal inputs or results to zero would be off by the
    whole value (thousands of units) in the second and third case."""
    A, B = operands(op, m, n, k, 990 + k)
    A = (A * np.float32(sa)).astype(np.float32)
    B = (B * np.float32(sb)).astype(np.float32)
    C, S = reference(op, A, B)
    got = run(op, -1, A, B).astype(np.float64)
    unit = 2.0 ** -149
    assert np.abs(C).max() > 1000 * unit, "the case must be far above the spacing, or a flush to zero would pass"
    if sa * sb > 2.0 ** -130 and k <= 64:
        want = C.astype(np.float32)
        assert ((want != 0) & (np.abs(want) < 2.0 ** -126)).mean() > 0.2, "the case must have subnormal results"
    excess = np.abs(got - C) - (k * unit + tol(k) * S)
    assert float(excess.max()) <= 0, f"off by {float(np.abs(got - C).max() / unit):.1f} units of 2^-149"
