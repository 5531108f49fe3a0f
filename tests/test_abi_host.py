"""Host-side tests of the C ABI: the library loads without a GPU, exports every declared symbol,
and rejects bad arguments before any device call (so fake pointers are safe here)."""
import ctypes
import os
import re

import pytest

from paper_1702_03192_amd import binding as mt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    return mt.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mtnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mtnn_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(L):
    names = declared_symbols()
    assert len(names) >= 20 and {"mtnn_nt", "mtnn_nn", "mtnn_transpose", "mtnn_select"} <= set(names)
    for name in names:
        assert hasattr(L, name), name
        assert name in mt.SIGNATURES, f"{name} has no binding signature"
    assert sorted(mt.SIGNATURES) == names


def test_version_and_status_strings(L):
    assert mt.mtnn_version() >= 100
    seen = {mt.mtnn_status_string(s) for s in range(10)}
    assert len(seen) == 10 and "ok" in seen
    assert mt.mtnn_status_string(1234) == "unknown status"


A, B, C, W = 0x100000, 0x200000, 0x300000, 0x400000   # fake device addresses, never dereferenced


def test_gemm_validation_codes(L):
    for fn in (L.mtnn_nt, L.mtnn_nn):
        assert fn(None, -1, 4, 4, A, 4, B, 4, C, 4) == 1
        assert fn(None, 4, 4, -2, A, 4, B, 4, C, 4) == 1
        assert fn(None, 4, 4, 4, None, 4, B, 4, C, 4) == 2
        assert fn(None, 4, 4, 4, A, 4, None, 4, C, 4) == 2
        assert fn(None, 4, 4, 4, A, 4, B, 4, None, 4) == 2
        assert fn(None, 4, 4, 8, A, 7, B, 8, C, 4) == 3      # lda < k
        assert fn(None, 4, 6, 4, A, 4, B, 8, C, 5) == 3      # ldc < n
        assert fn(None, 4, 4, 4, A, 4, B, 4, A + 16, 4) == 4  # C overlaps A
        assert fn(None, 4, 4, 4, A, 4, B, 4, B, 4) == 4       # C is B
        # empty problems succeed without touching anything (NULL pointers allowed)
        assert fn(None, 0, 4, 4, None, 4, None, 4, None, 4) == 0
        assert fn(None, 4, 0, 4, None, 4, None, 4, None, 4) == 0
    assert L.mtnn_nt(None, 4, 6, 8, A, 8, B, 7, C, 6) == 3    # NT: ldb < k
    assert L.mtnn_nn(None, 4, 6, 8, A, 8, B, 5, C, 6) == 3    # NN: ldb < n
    assert L.mtnn_nn(None, 4, 6, 8, A, 8, B, 6, C, 6) != 3


def test_ranges_use_leading_dimensions(L):
    # C starts right after the last logical element of A (A is 4 x 4 with lda 4 -> 64 bytes)
    assert L.mtnn_nt(None, 4, 4, 4, A, 4, B, 4, A + 60, 4) == 4
    # with lda = 8 the last row of A ends at byte (3*8+4)*4 = 112
    assert L.mtnn_nt(None, 4, 4, 4, A, 8, B, 4, A + 108, 4) == 4


def test_gemm_ex_arguments(L):
    n = L.mtnn_gemm_config_count()
    assert n >= 3
    assert L.mtnn_gemm_ex(None, 2, 0, 1, 4, 4, 4, A, 4, B, 4, C, 4) == 8
    assert L.mtnn_gemm_ex(None, 1, n, 1, 4, 4, 4, A, 4, B, 4, C, 4) == 8
    assert L.mtnn_gemm_ex(None, 1, -2, 1, 4, 4, 4, A, 4, B, 4, C, 4) == 8
    assert L.mtnn_gemm_ex(None, 1, 0, 33, 4, 4, 4, A, 4, B, 4, C, 4) == 8
    assert L.mtnn_gemm_ex(None, 1, 0, -1, 4, 4, 4, A, 4, B, 4, C, 4) == 8
    assert L.mtnn_gemm_ex(None, 1, 0, -3, 4, 4, 4, A, 4, B, 4, C, 4) == 8
    assert L.mtnn_gemm_ex(None, 1, 0, 1, 4, 4, 4, A, 3, B, 4, C, 4) == 3
    # the even cut is a legal request (validation goes on to the operands; an empty product is a success)
    assert mt.EVEN_CUT == -2
    assert L.mtnn_gemm_ex(None, 1, 0, mt.EVEN_CUT, 4, 4, 4, A, 3, B, 4, C, 4) == 3
    assert L.mtnn_gemm_ex(None, 1, 0, mt.EVEN_CUT, 0, 4, 4, A, 4, B, 4, C, 4) == 0
    assert mt.mtnn_gemm_even_cut_launches() >= 0
    names = mt.gemm_configs()
    assert len(set(names)) == n
    for op in (0, 1):
        for shape in [(256, 256, 256), (1024, 4096, 4096), (32, 8192, 8192), (8192, 32, 8192), (1000, 1000, 1000)]:
            assert 0 <= mt.mtnn_gemm_default_config(op, *shape) < n
            assert 1 <= mt.mtnn_gemm_default_splits(op, *shape) <= 32
        # an irregular mid-size shape with a long k is where the rule may answer "even cut"
        assert mt.mtnn_gemm_default_splits(op, 3000, 1500, 4500) in (mt.EVEN_CUT, 1, 2, 4)
    assert mt.mtnn_device_attribute(7) == -1          # unknown attribute
    assert mt.mtnn_gemm_default_config(0, 0, 4, 4) == -1


def test_fused_layer_calls_validation(L):
    Bias, W2 = 0x500000, 0x600000
    fwd = L.mtnn_fc_layer_forward
    ok_args = (4, 6, 8, A, 8, B, 8, Bias, 1, C, 6, W, 1 << 20, None)
    assert fwd(None, 2, *ok_args) == 8                                   # mode not in {-1, 0, +1}
    assert fwd(None, 1, 4, 6, 8, A, 8, B, 8, Bias, 2, C, 6, W, 1 << 20, None) == 8     # relu not 0 / 1
    assert fwd(None, 1, 4, 6, 8, A, 7, B, 8, Bias, 1, C, 6, W, 1 << 20, None) == 3     # ldx < k
    assert fwd(None, 1, 4, 6, 8, A, 8, B, 8, None, 1, C, 6, W, 1 << 20, None) == 2     # no bias
    assert fwd(None, 1, 4, 6, 8, A, 8, B, 8, C + 8, 1, C, 6, W, 1 << 20, None) == 4    # bias inside Y
    assert fwd(None, -1, 4, 6, 8, A, 8, B, 8, Bias, 1, C, 6, None, 0, None) == 5       # TNN without its workspace
    chosen = ctypes.c_int(0)
    assert fwd(None, 0, 0, 6, 8, None, 8, None, 8, None, 1, None, 6, None, 0, ctypes.byref(chosen)) == 0
    assert chosen.value == 1                                             # empty product: nothing to select
    upd = L.mtnn_fc_weight_grad_sgd
    assert upd(None, 4, 6, 8, A, 8, B, 5, C, 6, W2, 6, 0.1) == 3          # NN: ldb < n
    assert upd(None, 4, 6, 8, A, 8, B, 6, C, 6, None, 6, 0.1) == 2        # no W
    assert upd(None, 4, 6, 8, A, 8, B, 6, C, 6, W2, 5, 0.1) == 3          # ldw < n
    assert upd(None, 4, 6, 8, A, 8, B, 6, C, 6, C + 16, 6, 0.1) == 4      # W overlaps dW
    assert upd(None, 4, 6, 8, A, 8, B, 6, C, 6, A, 6, 0.1) == 4           # W is A
    assert upd(None, 0, 6, 8, None, 8, None, 6, None, 6, None, 6, 0.1) == 0
    assert L.mtnn_gemm_fused_epilogue_launches() >= 0
    assert L.mtnn_set_fused_epilogues(0) == 1 and L.mtnn_set_fused_epilogues(1) == 0 and L.mtnn_set_fused_epilogues(1) == 1


def test_transpose_validation_codes(L):
    assert L.mtnn_transpose(None, -1, 4, A, 4, B, 4) == 1
    assert L.mtnn_transpose(None, 4, 6, None, 6, B, 4) == 2
    assert L.mtnn_transpose(None, 4, 6, A, 5, B, 4) == 3     # ldin < cols
    assert L.mtnn_transpose(None, 4, 6, A, 6, B, 3) == 3     # ldout < rows
    assert L.mtnn_transpose(None, 4, 6, A, 6, A, 4) == 4     # in place is not supported
    assert L.mtnn_transpose(None, 0, 6, None, 6, None, 1) == 0
    assert L.mtnn_transpose(None, 4, 0, None, 1, None, 4) == 0


def test_tnn_workspace_rules(L):
    assert mt.mtnn_tnn_workspace_bytes(0, 5) == 0 and mt.mtnn_tnn_workspace_bytes(5, -1) == 0
    assert mt.mtnn_tnn_workspace_bytes(3, 5) == 256                 # 60 B rounded up
    assert mt.mtnn_tnn_workspace_bytes(8192, 8192) == 8192 * 8192 * 4
    assert mt.mtnn_tnn_workspace_bytes(65536, 65536) == 65536 * 65536 * 4   # no 32-bit overflow
    need = mt.mtnn_tnn_workspace_bytes(6, 8)
    assert L.mtnn_tnn(None, 4, 6, 8, A, 8, B, 8, C, 6, None, 0) == 5
    assert L.mtnn_tnn(None, 4, 6, 8, A, 8, B, 8, C, 6, W, need - 1) == 5
    assert L.mtnn_tnn(None, 4, 6, 8, A, 8, B, 8, C, 6, B + 8, need) == 4     # workspace overlaps B
    assert L.mtnn_tnn(None, 4, 6, 8, A, 7, B, 8, C, 6, W, need) == 3         # argument checks come first
    assert L.mtnn_tnn(None, 0, 6, 8, None, 8, None, 8, None, 6, None, 0) == 0
    chosen = ctypes.c_int(7)
    assert L.mtnn_auto(None, 4, 6, 8, A, 7, B, 8, C, 6, W, need, ctypes.byref(chosen)) == 3


def test_fc_step_validation(L):
    import ctypes
    dims = (ctypes.c_int * 3)(8, 16, 4)
    assert L.mtnn_fc_workspace_bytes(0, dims, 4) == 0
    assert L.mtnn_fc_workspace_bytes(2, dims, 0) == 0
    need = L.mtnn_fc_workspace_bytes(2, dims, 4)
    # H1 4x16, H2 4x4, dA, dB 4x16 each, dZt 16x4, Bt 16x8, row_loss 4 (each rounded to 256 B), bias partials 32x16
    assert need == 256 + 256 + 2 * 256 + 256 + 512 + 256 + 2048
    assert L.mtnn_fc_train_step(None, None) == 2
    ptrs = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    d = mt.FcStepDesc(2, dims, 4, 0x100, 0x200, ptrs, ptrs, ptrs, ptrs, None, 0x300, 0x400, need - 1, 0.01, 0)
    assert L.mtnn_fc_train_step(None, ctypes.byref(d)) == 5            # workspace too small
    d.workspace_bytes = need
    d.forward_mode = 3
    assert L.mtnn_fc_train_step(None, ctypes.byref(d)) == 8
    d.forward_mode = 0
    d.X = None
    assert L.mtnn_fc_train_step(None, ctypes.byref(d)) == 2
    d.X = 0x100
    d.batch = 0
    assert L.mtnn_fc_train_step(None, ctypes.byref(d)) == 1
    assert L.mtnn_fc_sgd(None, -1, 0x10, 0x20, 0.1) == 1
    assert L.mtnn_fc_bias_act(None, 4, 4, None, 0x20, 1) == 2


def test_inplace_transpose_validation(L):
    assert L.mtnn_transpose_inplace(None, -1, A, 4) == 1
    assert L.mtnn_transpose_inplace(None, 4, None, 4) == 2
    assert L.mtnn_transpose_inplace(None, 4, A, 3) == 3
    assert L.mtnn_transpose_inplace(None, 0, None, 0) == 0
    assert L.mtnn_tnn_inplace(None, 4, 6, 8, A, 9, B, 9, C, 6) == 8      # B rectangular and not dense
    assert L.mtnn_tnn_inplace(None, 4, 40000, 8, A, 8, B, 8, 0x40000000, 40000) == 8   # beyond the in-place kernel's limit
    assert L.mtnn_tnn_inplace(None, 4, 6, 8, A, 8, B, 8, C, 6) in (0, 9)  # dense rectangular B: accepted
    assert L.mtnn_tnn_inplace_supported(6, 8, 8) == 1 and L.mtnn_tnn_inplace_supported(6, 8, 9) == 0
    assert L.mtnn_tnn_inplace_supported(8, 8, 11) == 1 and L.mtnn_tnn_inplace_supported(8, 8, 7) == 0
    assert L.mtnn_tnn_inplace_supported(32768, 5, 5) == 1 and L.mtnn_tnn_inplace_supported(32769, 5, 5) == 0
    assert L.mtnn_transpose_inplace_rect(None, -1, 4, A) == 1
    assert L.mtnn_transpose_inplace_rect(None, 4, 6, None) == 2
    assert L.mtnn_transpose_inplace_rect(None, 4, 40000, A) == 8
    assert L.mtnn_transpose_inplace_rect(None, 0, 6, None) == 0
    assert L.mtnn_transpose_inplace_rect(None, 1, 60000, A) == 0          # a vector: nothing to move
    assert L.mtnn_tnn_inplace(None, 4, 8, 8, A, 7, B, 8, C, 8) == 3


def test_cost_model_choice_is_valid_and_repeatable_over_many_shapes():
    """The configuration / split rule on 3000 seeded shapes from 1 to 2^17 per dimension (pure host code):
    always a configuration of the table and a split count the launcher accepts, the same on every call,
    and split-k only where every split keeps at least 128 of k."""
    import numpy as np
    rng = np.random.default_rng(1702)
    n_cfg = len(mt.gemm_configs())
    dims = np.exp(rng.uniform(0.0, np.log(2.0 ** 17), size=(3000, 3))).astype(np.int64)
    dims[:8] = [[1, 1, 1], [1, 131072, 1], [131072, 1, 131072], [65536, 65536, 65536], [1, 1, 131072],
                [131072, 131072, 1], [7, 5, 3], [255, 257, 129]]
    for m, n, k in dims:
        m, n, k = int(m), int(n), int(k)
        for op in (0, 1):
            c, s = mt.mtnn_gemm_default_config(op, m, n, k), mt.mtnn_gemm_default_splits(op, m, n, k)
            assert 0 <= c < n_cfg
            assert s == mt.EVEN_CUT or s in (1, 2, 4, 8, 16, 32)
            if s > 1:
                assert k // s >= 128 and m * n * s * 4 <= (64 << 20)
            assert (c, s) == (mt.mtnn_gemm_default_config(op, m, n, k), mt.mtnn_gemm_default_splits(op, m, n, k))


def test_no_device_is_reported_not_a_launch_error(L):
    """Without a usable gfx950 (this test runs where there is no GPU at all) a call with valid arguments
    launches nothing and says so; validation errors still come first."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    assert L.mtnn_nt(None, 4, 6, 8, A, 8, B, 8, C, 6) == 9
    assert L.mtnn_nn(None, 4, 6, 8, A, 8, B, 6, C, 6) == 9
    assert L.mtnn_nt(None, 4, 6, 0, None, 1, None, 1, C, 6) == 9          # k = 0 still has to write zeros
    assert L.mtnn_transpose(None, 4, 6, A, 6, B, 4) == 9
    assert L.mtnn_transpose_inplace(None, 4, A, 4) == 9
    assert L.mtnn_copy_bytes(None, 64, A, B) == 9
    assert L.mtnn_tnn(None, 4, 6, 8, A, 8, B, 8, C, 6, W, 256) == 9
    assert L.mtnn_nt(None, 4, 6, 8, A, 7, B, 8, C, 6) == 3                # a bad argument is still a bad argument
    assert L.mtnn_set_scratch(None, 0x700000, 1 << 20) == 9               # scratch belongs to a device's stream
    assert L.mtnn_get_scratch_bytes(None) == 0
    assert "gfx950" in mt.mtnn_status_string(9)


def test_architecture_test_on_names(L):
    ok = [b"gfx950", b"gfx950:sramecc+:xnack-", b"gfx950:xnack-"]
    bad = [b"gfx942", b"gfx942:sramecc+:xnack-", b"gfx90a", b"gfx9500", b"gfx95", b"", b"sm_90", b"gfx1100"]
    assert all(L.mtnn_arch_supported(a) == 1 for a in ok)
    assert all(L.mtnn_arch_supported(a) == 0 for a in bad)
    assert L.mtnn_arch_supported(None) == 0


def test_scratch_arguments_and_needs(L):
    assert L.mtnn_set_scratch(None, None, 64) == 8                         # bytes without memory
    assert L.mtnn_set_scratch(None, 0x700000, 0) == 8                      # memory without bytes
    assert L.mtnn_set_scratch(None, 0x700010, 1 << 20) == 8                # not 256-byte aligned
    assert L.mtnn_scratch_bytes_default() == 64 << 20
    assert mt.mtnn_gemm_scratch_bytes(3, 4, 100, 200, 4096) == 100 * 200 * 4 * 4
    assert mt.mtnn_gemm_scratch_bytes(3, 32, 100, 200, 130) == 100 * 200 * 4 * 3   # empty splits are dropped: 3 ranges of 64
    assert mt.mtnn_gemm_scratch_bytes(3, 1, 100, 200, 4096) == 0
    assert mt.mtnn_gemm_scratch_bytes(99, 4, 100, 200, 4096) == 0
    # the even cut: two tile-sized slots per workgroup of the fixed grid (nominal device: 256 CUs x 2 per CU)
    assert mt.mtnn_gemm_scratch_bytes(10, mt.EVEN_CUT, 1000, 900, 1100) == 2 * 512 * 128 * 128 * 4


def test_choice_respects_the_scratch_capacity():
    """The cost model only considers divisions whose partial products fit the scratch it is told about."""
    import numpy as np
    rng = np.random.default_rng(3192)
    dims = np.exp(rng.uniform(np.log(16.0), np.log(2.0 ** 14), size=(400, 3))).astype(np.int64)
    n_cfg = len(mt.gemm_configs())
    saw_split = False
    for m, n, k in dims:
        m, n, k = int(m), int(n), int(k)
        for op in (0, 1):
            assert mt.mtnn_gemm_choice(op, m, n, k, 0)[1] == 1             # no scratch: unsplit launches only
            for cap in (1 << 16, 1 << 22, 64 << 20):
                c, s = mt.mtnn_gemm_choice(op, m, n, k, cap)
                assert 0 <= c < n_cfg
                if s != 1:
                    saw_split = True
                    assert 0 < mt.mtnn_gemm_scratch_bytes(c, s, m, n, k) <= cap
            assert mt.mtnn_gemm_choice(op, m, n, k) == (mt.mtnn_gemm_default_config(op, m, n, k),
                                                        mt.mtnn_gemm_default_splits(op, m, n, k))
    assert saw_split


def test_two_wave_set_configurations_are_chosen_where_a_cu_holds_one_workgroup():
    """Configurations whose workgroups run two sets of waves on one tile ("k2" in the name) are for
    launches of at most one workgroup per CU with 512-2048 k each; the 32-row / 32-column ones only for
    products one tile high / wide."""
    names = mt.gemm_configs()
    k2 = lambda op, m, n, k: "k2" in names[mt.mtnn_gemm_choice(op, m, n, k)[0]]
    for op in (0, 1):
        assert k2(op, 1024, 1024, 1024) and k2(op, 2048, 512, 1024)          # 256 tiles of 64 x 64
        assert k2(op, 32, 8192, 8192) and k2(op, 8192, 32, 8192)             # one tile high / wide, split-k
        assert names[mt.mtnn_gemm_choice(op, 32, 8192, 8192)[0]].startswith("32x256")
        assert names[mt.mtnn_gemm_choice(op, 8192, 32, 8192)[0]].startswith("256x32")
        assert not k2(op, 8192, 8192, 8192) and not k2(op, 4096, 4096, 1024)  # many workgroups per CU
        assert not k2(op, 1024, 1024, 64) and not k2(op, 256, 256, 256)      # too little k per workgroup
        assert not k2(op, 64, 8192, 8192)                                    # two tiles high: not the skinny tile
    import numpy as np
    rng = np.random.default_rng(1702)
    for m, n, k in np.exp(rng.uniform(np.log(16.0), np.log(2.0 ** 14), size=(300, 3))).astype(np.int64):
        for op in (0, 1):
            c, s = mt.mtnn_gemm_choice(op, int(m), int(n), int(k))
            if "k2" in names[c]:
                bm, bn = (int(v) for v in names[c].split("x")[:2])
                assert s >= 1 and -(-int(m) // bm) * -(-int(n) // bn) * s <= 256 and 512 <= int(k) // s <= 2048


def test_tnn_inplace_rejects_b_overlapping_a(L):
    """B is written by the in-place path, so the Gram product A x A^T (A == B) must be refused."""
    assert L.mtnn_tnn_inplace(None, 8, 8, 8, A, 8, A, 8, C, 8) == 4
    assert L.mtnn_tnn_inplace(None, 4, 8, 8, A + 32 * 4, 8, A, 8, C, 8) == 4      # A inside B
    assert L.mtnn_tnn_inplace(None, 8, 8, 8, A, 8, B, 8, C, 8) in (0, 6, 9)       # disjoint: passes validation


def test_three_way_choice_validation_and_rule(L):
    need = mt.mtnn_tnn_workspace_bytes(6, 8)
    chosen = ctypes.c_int(9)
    assert L.mtnn_auto3(None, 2, 4, 6, 8, A, 8, B, 8, C, 6, W, need, ctypes.byref(chosen)) == 8      # unknown mode
    assert L.mtnn_auto3(None, 0, 4, 6, 8, A, 7, B, 8, C, 6, W, need, ctypes.byref(chosen)) == 3      # argument checks first
    assert L.mtnn_auto3(None, -1, 4, 6, 8, A, 8, B, 8, C, 6, None, 0, ctypes.byref(chosen)) == 5     # forced TNN needs its workspace
    assert chosen.value == -1
    assert L.mtnn_auto3(None, -2, 4, 6, 8, A, 8, B, 9, C, 6, None, 0, ctypes.byref(chosen)) == 8     # forced in-place, B not dense
    assert L.mtnn_auto3(None, -2, 8, 8, 8, A, 8, A, 8, C, 8, None, 0, ctypes.byref(chosen)) == 4     # ... and B must not be A
    assert L.mtnn_auto3(None, 0, 0, 6, 8, None, 8, None, 8, None, 6, None, 0, ctypes.byref(chosen)) == 0
    assert chosen.value == 1
    # the rule: NT where the predictor says NT; TNN where it says TNN and there is room; without room, in place only if allowed and worth it
    assert L.mtnn_select3(0, 4, 4, 1, 1) == 0
    rows = [(m, n, k) for m in (64, 512, 4096) for n in (64, 512, 4096) for k in (64, 512, 4096)]
    try:
        mt.mtnn_train_selector(rows, [1] * len(rows))
        assert all(L.mtnn_select3(m, n, k, w, ip) == 1 for m, n, k in rows for w in (0, 1) for ip in (0, 1))
        mt.mtnn_train_selector(rows, [-1] * len(rows))
        for m, n, k in rows:
            assert L.mtnn_select(m, n, k) == -1
            assert L.mtnn_select3(m, n, k, 1, 0) == -1 and L.mtnn_select3(m, n, k, 1, 1) == -1
            assert L.mtnn_select3(m, n, k, 0, 0) == 1                      # the memory rule of Section II
            assert L.mtnn_select3(m, n, k, 0, 1) in (1, -2)
        # the two kernels are tuned alike here, so two more passes over B never pay on these shapes
        assert all(L.mtnn_select3(m, n, k, 0, 1) == 1 for m, n, k in rows)
    finally:
        mt.mtnn_unload_model()
        if os.path.exists(mt.DEFAULT_MODEL):
            mt.mtnn_load_model(mt.DEFAULT_MODEL)
