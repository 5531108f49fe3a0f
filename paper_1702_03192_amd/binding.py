"""Thin ctypes binding of libmtnn.so: same names as the C ABI, argument marshalling only.

Device buffers are torch tensors (PyTorch owns device memory and streams); every step of the
path runs inside the library's HIP kernels.  There is no CPU fallback: if the library has not
been built the import of any entry point raises.
"""
from __future__ import annotations

import ctypes
import threading
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmtnn.so")
DEFAULT_MODEL = os.path.join(HERE, "data", "selector_gfx950.model")

OK = 0
STATUS_NAMES = {0: "OK", 1: "ERR_DIM", 2: "ERR_NULL", 3: "ERR_LD", 4: "ERR_ALIAS", 5: "ERR_WORKSPACE",
                6: "ERR_LAUNCH", 7: "ERR_MODEL", 8: "ERR_ARG", 9: "ERR_NO_DEVICE"}
OP_NN, OP_NT = 0, 1

_c_int = ctypes.c_int
_c_vp = ctypes.c_void_p
_c_sz = ctypes.c_size_t
_c_dbl = ctypes.c_double
_p_int = ctypes.POINTER(ctypes.c_int)
_p_dbl = ctypes.POINTER(ctypes.c_double)

_c_ll = ctypes.c_longlong
_c_flt = ctypes.c_float


class FcStepDesc(ctypes.Structure):
    """Mirror of mtnn_fc_step_desc."""
    _fields_ = [("num_layers", _c_int), ("dims", _p_int), ("batch", _c_int), ("X", _c_vp), ("labels", _c_vp),
                ("W", ctypes.POINTER(_c_vp)), ("b", ctypes.POINTER(_c_vp)), ("dW", ctypes.POINTER(_c_vp)),
                ("db", ctypes.POINTER(_c_vp)), ("logits", _c_vp), ("loss", _c_vp), ("workspace", _c_vp),
                ("workspace_bytes", _c_sz), ("lr", _c_flt), ("forward_mode", _c_int)]


_GEMM = [_c_vp, _c_int, _c_int, _c_int, _c_vp, _c_int, _c_vp, _c_int, _c_vp, _c_int]

# name -> (restype, argtypes): every symbol include/mtnn.h declares
SIGNATURES = {
    "mtnn_nt": (_c_int, _GEMM),
    "mtnn_nn": (_c_int, _GEMM),
    "mtnn_transpose": (_c_int, [_c_vp, _c_int, _c_int, _c_vp, _c_int, _c_vp, _c_int]),
    "mtnn_transpose_inplace": (_c_int, [_c_vp, _c_int, _c_vp, _c_int]),
    "mtnn_tnn_inplace": (_c_int, _GEMM),
    "mtnn_tnn_inplace_supported": (_c_int, [_c_int, _c_int, _c_int]),
    "mtnn_transpose_inplace_rect": (_c_int, [_c_vp, _c_int, _c_int, _c_vp]),
    "mtnn_select3": (_c_int, [_c_int, _c_int, _c_int, _c_int, _c_int]),
    "mtnn_auto3": (_c_int, [_c_vp, _c_int] + _GEMM[1:] + [_c_vp, _c_sz, _p_int]),
    "mtnn_tnn_workspace_bytes": (_c_sz, [_c_int, _c_int]),
    "mtnn_tnn": (_c_int, _GEMM + [_c_vp, _c_sz]),
    "mtnn_auto": (_c_int, _GEMM + [_c_vp, _c_sz, _p_int]),
    "mtnn_select": (_c_int, [_c_int, _c_int, _c_int]),
    "mtnn_select_batch": (_c_int, [_c_int, _c_vp, _c_vp]),
    "mtnn_num_features": (_c_int, []),
    "mtnn_features": (_c_int, [_c_int, _c_int, _c_int, _p_dbl]),
    "mtnn_load_model": (_c_int, [ctypes.c_char_p]),
    "mtnn_save_model": (_c_int, [ctypes.c_char_p]),
    "mtnn_unload_model": (None, []),
    "mtnn_gbdt_train": (_c_int, [_c_int, _c_int, _c_vp, _c_vp, _c_int, _c_int, _c_dbl, _c_dbl, _c_dbl, _c_dbl]),
    "mtnn_train_selector": (_c_int, [_c_int, _c_vp, _c_vp]),
    "mtnn_model_num_trees": (_c_int, []),
    "mtnn_model_num_features": (_c_int, []),
    "mtnn_model_tree_size": (_c_int, [_c_int]),
    "mtnn_model_node": (_c_int, [_c_int, _c_int, _p_int, _p_dbl, _p_int, _p_int, _p_dbl]),
    "mtnn_model_margin": (_c_int, [_c_vp, _c_int, _p_dbl]),
    "mtnn_gemm_config_count": (_c_int, []),
    "mtnn_gemm_config_name": (ctypes.c_char_p, [_c_int]),
    "mtnn_gemm_default_config": (_c_int, [_c_int, _c_int, _c_int, _c_int]),
    "mtnn_gemm_default_splits": (_c_int, [_c_int, _c_int, _c_int, _c_int]),
    "mtnn_gemm_ex": (_c_int, [_c_vp, _c_int, _c_int, _c_int] + _GEMM[1:]),
    "mtnn_gemm_ex_static": (_c_int, [_c_vp, _c_int, _c_int, _c_int] + _GEMM[1:]),
    "mtnn_set_scratch": (_c_int, [_c_vp, _c_vp, _c_sz]),
    "mtnn_get_scratch_bytes": (_c_sz, [_c_vp]),
    "mtnn_scratch_bytes_default": (_c_sz, []),
    "mtnn_gemm_scratch_bytes": (_c_sz, [_c_int, _c_int, _c_int, _c_int, _c_int]),
    "mtnn_gemm_choice": (_c_int, [_c_int, _c_int, _c_int, _c_int, _c_sz, _p_int, _p_int]),
    "mtnn_arch_supported": (_c_int, [ctypes.c_char_p]),
    "mtnn_fc_workspace_bytes": (_c_sz, [_c_int, _p_int, _c_int]),
    "mtnn_fc_train_step": (_c_int, [_c_vp, ctypes.POINTER(FcStepDesc)]),
    "mtnn_fc_forward": (_c_int, [_c_vp, ctypes.POINTER(FcStepDesc)]),
    "mtnn_fc_bias_act": (_c_int, [_c_vp, _c_int, _c_int, _c_vp, _c_vp, _c_int]),
    "mtnn_fc_softmax_xent": (_c_int, [_c_vp, _c_int, _c_int, _c_vp, _c_vp, _c_vp, _c_vp, _c_vp]),
    "mtnn_fc_relu_backward": (_c_int, [_c_vp, _c_ll, _c_vp, _c_vp]),
    "mtnn_fc_bias_grad": (_c_int, [_c_vp, _c_int, _c_int, _c_vp, _c_vp, _c_vp]),
    "mtnn_fc_relu_backward_bias_grad": (_c_int, [_c_vp, _c_int, _c_int, _c_vp, _c_vp, _c_vp, _c_vp]),
    "mtnn_fc_sgd": (_c_int, [_c_vp, _c_ll, _c_vp, _c_vp, _c_flt]),
    "mtnn_fc_layer_forward": (_c_int, [_c_vp, _c_int, _c_int, _c_int, _c_int, _c_vp, _c_int, _c_vp, _c_int, _c_vp, _c_int,
                                       _c_vp, _c_int, _c_vp, _c_sz, _p_int]),
    "mtnn_fc_weight_grad_sgd": (_c_int, [_c_vp, _c_int, _c_int, _c_int, _c_vp, _c_int, _c_vp, _c_int, _c_vp, _c_int,
                                         _c_vp, _c_int, _c_flt]),
    "mtnn_copy_rows": (_c_int, [_c_vp, _c_int, _c_int, _c_vp, _c_vp]),
    "mtnn_copy_bytes": (_c_int, [_c_vp, _c_sz, _c_vp, _c_vp]),
    "mtnn_probe_lanes": (_c_int, [_c_vp, _c_int, _c_int, _c_vp]),
    "mtnn_status_string": (ctypes.c_char_p, [_c_int]),
    "mtnn_last_hip_error": (_c_int, []),
    "mtnn_version": (_c_int, []),
    "mtnn_gemm_even_cut_launches": (ctypes.c_longlong, []),
    "mtnn_gemm_fused_epilogue_launches": (ctypes.c_longlong, []),
    "mtnn_set_fused_epilogues": (_c_int, [_c_int]),
    "mtnn_device_attribute": (_c_int, [_c_int]),
}

_lib = None


class MtnnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({STATUS_NAMES.get(status, '?')})")


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_1702_03192_amd.build` "
                               "(or __graft_entry__.build()) first; there is no CPU fallback")
        # torch first: the library shares the HIP runtime torch has loaded (one runtime per
        # process, so torch's streams and allocations are valid inside the library)
        import torch  # noqa: F401
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
        if os.path.exists(DEFAULT_MODEL) and not os.environ.get("MTNN_NO_DEFAULT_MODEL"):
            handle.mtnn_load_model(DEFAULT_MODEL.encode())
    return _lib


def _check(status: int, where: str) -> None:
    if status != OK:
        if status == 6:
            where = f"{where} (hipError {lib().mtnn_last_hip_error()})"
        raise MtnnError(status, where)


# The library allocates nothing: launches that divide a product over several workgroups per C tile
# keep their partial products in scratch memory lent per (device, stream).  This binding lends a torch
# tensor of the default capacity the first time it sees a stream, so that every call on that stream
# -- eager or under capture -- is divided the same way.
_scratch = {}     # (device index, stream handle) -> the tensor lent to the library


def lend_scratch(stream=None, nbytes: Optional[int] = None):
    """Lend the library `nbytes` (default: mtnn_scratch_bytes_default()) of scratch for `stream` of the current
    device, replacing what was lent before.  nbytes = 0 withdraws it (split launches then do not run)."""
    import torch
    h = _handle(stream)
    key = (torch.cuda.current_device(), h)
    if nbytes is None:
        nbytes = int(lib().mtnn_scratch_bytes_default())
    if nbytes == 0:
        _check(lib().mtnn_set_scratch(h or None, None, 0), "mtnn_set_scratch")
        _scratch[key] = None
        return None
    if torch.cuda.is_current_stream_capturing():
        raise RuntimeError("scratch cannot be allocated while a stream is being captured: call lend_scratch(stream) "
                           "(or run one call on the stream) before the capture begins")
    buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    _check(lib().mtnn_set_scratch(h or None, buf.data_ptr(), nbytes), "mtnn_set_scratch")
    _scratch[key] = buf      # (the previous tensor, if any, is released only now that the library no longer points at it)
    return buf


def _handle(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


def _stream(stream) -> Optional[int]:
    import torch
    h = _handle(stream)
    if (torch.cuda.current_device(), h) not in _scratch:
        lend_scratch(h)
    return h or None


def _dev(t, name):
    """(pointer, leading dimension) of a 2-D fp32 device tensor whose rows are contiguous."""
    import torch
    if t.dtype != torch.float32 or t.dim() != 2 or not t.is_cuda:
        raise TypeError(f"{name} must be a 2-D float32 device tensor")
    if t.shape[1] > 1 and t.stride(1) != 1:
        raise TypeError(f"{name} must have unit column stride")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], 1)
    return t.data_ptr(), int(ld)


_tls = threading.local()      # per-thread out-parameter of mtnn_auto, allocated once


def _ws(workspace):
    if workspace is None:
        return None, 0
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


# ---- dense operations: the tensors' shapes give m, n, k and the leading dimensions -----------

def mtnn_nt(A, B, C, stream=None):
    """C = A x B^T.  A: m x k, B: n x k, C: m x n."""
    (pa, lda), (pb, ldb), (pc, ldc) = _dev(A, "A"), _dev(B, "B"), _dev(C, "C")
    m, k = A.shape
    n = B.shape[0]
    if B.shape[1] != k or tuple(C.shape) != (m, n):
        raise ValueError("shape mismatch")
    _check(lib().mtnn_nt(_stream(stream), m, n, k, pa, lda, pb, ldb, pc, ldc), "mtnn_nt")
    return C


def mtnn_nn(A, B, C, stream=None):
    """C = A x B.  A: m x k, B: k x n, C: m x n."""
    (pa, lda), (pb, ldb), (pc, ldc) = _dev(A, "A"), _dev(B, "B"), _dev(C, "C")
    m, k = A.shape
    n = B.shape[1]
    if B.shape[0] != k or tuple(C.shape) != (m, n):
        raise ValueError("shape mismatch")
    _check(lib().mtnn_nn(_stream(stream), m, n, k, pa, lda, pb, ldb, pc, ldc), "mtnn_nn")
    return C


def mtnn_gemm_ex(op, cfg, A, B, C, stream=None, splits=0):
    """A given tile configuration / split count of the NN (op 0) or NT (op 1) kernel; cfg -1 = default rule."""
    (pa, lda), (pb, ldb), (pc, ldc) = _dev(A, "A"), _dev(B, "B"), _dev(C, "C")
    m, k = A.shape
    n = B.shape[0] if op == OP_NT else B.shape[1]
    _check(lib().mtnn_gemm_ex(_stream(stream), op, cfg, splits, m, n, k, pa, lda, pb, ldb, pc, ldc), "mtnn_gemm_ex")
    return C


def mtnn_gemm_ex_static(op, cfg, A, B, C, stream=None, splits=0):
    """mtnn_gemm_ex with the library's own static scratch (32 MiB per GPU): allocates nothing."""
    (pa, lda), (pb, ldb), (pc, ldc) = _dev(A, "A"), _dev(B, "B"), _dev(C, "C")
    m, k = A.shape
    n = B.shape[0] if op == OP_NT else B.shape[1]
    _check(lib().mtnn_gemm_ex_static(_handle(stream) or None, op, cfg, splits, m, n, k, pa, lda, pb, ldb, pc, ldc),
           "mtnn_gemm_ex_static")
    return C


def mtnn_transpose(X, out, stream=None):
    """out = X^T, bit-exact.  X: rows x cols, out: cols x rows."""
    (pi, ldi), (po, ldo) = _dev(X, "in"), _dev(out, "out")
    rows, cols = X.shape
    if tuple(out.shape) != (cols, rows):
        raise ValueError("shape mismatch")
    _check(lib().mtnn_transpose(_stream(stream), rows, cols, pi, ldi, po, ldo), "mtnn_transpose")
    return out


def mtnn_transpose_inplace(X, stream=None):
    """X <- X^T for a square matrix, in place, bit-exact."""
    p, ld = _dev(X, "X")
    if X.shape[0] != X.shape[1]:
        raise ValueError("square matrices only")
    _check(lib().mtnn_transpose_inplace(_stream(stream), X.shape[0], p, ld), "mtnn_transpose_inplace")
    return X


def mtnn_transpose_inplace_rect(X, rows: int, cols: int, stream=None):
    """The dense rows x cols matrix in the 1-D (or any contiguous) tensor X becomes cols x rows, in place."""
    if not X.is_contiguous() or X.numel() != rows * cols:
        raise ValueError("X must be a contiguous tensor of rows * cols elements")
    _check(lib().mtnn_transpose_inplace_rect(_stream(stream), rows, cols, X.data_ptr()), "mtnn_transpose_inplace_rect")
    return X


def mtnn_select3(m: int, n: int, k: int, have_workspace: bool, can_inplace: bool) -> int:
    return int(lib().mtnn_select3(m, n, k, int(have_workspace), int(can_inplace)))


def mtnn_auto3(A, B, C, workspace=None, mode: int = 0, stream=None) -> int:
    """NT (+1), TNN (-1) or TNN through in-place transposes of B (-2): the rule (mode 0) or a forced path."""
    (pa, lda), (pb, ldb), (pc, ldc) = _dev(A, "A"), _dev(B, "B"), _dev(C, "C")
    m, k = A.shape
    n = B.shape[0]
    pw, wb = _ws(workspace)
    chosen = ctypes.c_int(0)
    _check(lib().mtnn_auto3(_stream(stream), mode, m, n, k, pa, lda, pb, ldb, pc, ldc, pw, wb, ctypes.byref(chosen)),
           "mtnn_auto3")
    return chosen.value


def mtnn_tnn_inplace(A, B, C, stream=None):
    """C = A x B^T through in-place transposes of B (restored afterwards)."""
    (pa, lda), (pb, ldb), (pc, ldc) = _dev(A, "A"), _dev(B, "B"), _dev(C, "C")
    m, k = A.shape
    n = B.shape[0]
    _check(lib().mtnn_tnn_inplace(_stream(stream), m, n, k, pa, lda, pb, ldb, pc, ldc), "mtnn_tnn_inplace")
    return C


def mtnn_tnn_workspace_bytes(n: int, k: int) -> int:
    return int(lib().mtnn_tnn_workspace_bytes(n, k))


def mtnn_tnn(A, B, C, workspace, stream=None):
    """Algorithm 1 with a caller-owned B^T workspace (any device tensor of enough bytes)."""
    (pa, lda), (pb, ldb), (pc, ldc) = _dev(A, "A"), _dev(B, "B"), _dev(C, "C")
    m, k = A.shape
    n = B.shape[0]
    pw, wb = _ws(workspace)
    _check(lib().mtnn_tnn(_stream(stream), m, n, k, pa, lda, pb, ldb, pc, ldc, pw, wb), "mtnn_tnn")
    return C


def mtnn_auto(A, B, C, workspace=None, stream=None) -> int:
    """Algorithm 2.  Returns the label of the path that ran (+1 NT, -1 TNN)."""
    (pa, lda), (pb, ldb), (pc, ldc) = _dev(A, "A"), _dev(B, "B"), _dev(C, "C")
    m, k = A.shape
    n = B.shape[0]
    pw, wb = _ws(workspace)
    chosen = getattr(_tls, "chosen", None)
    if chosen is None:
        chosen = _tls.chosen = ctypes.c_int(0)
        _tls.chosen_ref = ctypes.byref(chosen)
    _check(lib().mtnn_auto(_stream(stream), m, n, k, pa, lda, pb, ldb, pc, ldc, pw, wb, _tls.chosen_ref), "mtnn_auto")
    return chosen.value


# ---- prepared calls ------------------------------------------------------------------------

class Prepared:
    """One library call with every argument resolved beforehand: pointers, leading dimensions, sizes and
    the stream are taken from the tensors once, so that calling the object is a single ctypes call.
    For loops that issue the same call many times (training steps, timing batches): the wrappers above
    spend several microseconds per call on tensor checks and the stream lookup, which is more than a
    small product takes on the GPU.  The object keeps its tensors alive; it must not outlive the
    stream it was prepared for."""
    __slots__ = ("_fn", "_args", "_name", "_keep", "_chosen")

    def __init__(self, name, args, keep, chosen=None):
        self._fn = getattr(lib(), name)
        self._args = args
        self._name = name
        self._keep = keep
        self._chosen = chosen

    def __call__(self):
        status = self._fn(*self._args)
        if status:
            _check(status, self._name)
        return self._chosen.value if self._chosen is not None else None


def _gemm_args(op, A, B, C, stream):
    (pa, lda), (pb, ldb), (pc, ldc) = _dev(A, "A"), _dev(B, "B"), _dev(C, "C")
    m, k = A.shape
    n = B.shape[0] if op == OP_NT else B.shape[1]
    if (B.shape[1] if op == OP_NT else B.shape[0]) != k or tuple(C.shape) != (m, n):
        raise ValueError("shape mismatch")
    return (_stream(stream), m, n, k, pa, lda, pb, ldb, pc, ldc)


def prepare_nt(A, B, C, stream=None) -> Prepared:
    return Prepared("mtnn_nt", _gemm_args(OP_NT, A, B, C, stream), (A, B, C))


def prepare_nn(A, B, C, stream=None) -> Prepared:
    return Prepared("mtnn_nn", _gemm_args(OP_NN, A, B, C, stream), (A, B, C))


def prepare_gemm_ex(op, cfg, A, B, C, stream=None, splits=0) -> Prepared:
    a = _gemm_args(op, A, B, C, stream)
    return Prepared("mtnn_gemm_ex", (a[0], op, cfg, splits) + a[1:], (A, B, C))


def prepare_tnn(A, B, C, workspace, stream=None) -> Prepared:
    pw, wb = _ws(workspace)
    return Prepared("mtnn_tnn", _gemm_args(OP_NT, A, B, C, stream) + (pw, wb), (A, B, C, workspace))


def prepare_auto(A, B, C, workspace=None, stream=None) -> Prepared:
    """Calling the result runs Algorithm 2 and returns the label of the path taken."""
    pw, wb = _ws(workspace)
    chosen = ctypes.c_int(0)
    return Prepared("mtnn_auto", _gemm_args(OP_NT, A, B, C, stream) + (pw, wb, ctypes.byref(chosen)),
                    (A, B, C, workspace), chosen)


def prepare_transpose(X, out, stream=None) -> Prepared:
    (pi, ldi), (po, ldo) = _dev(X, "in"), _dev(out, "out")
    rows, cols = X.shape
    if tuple(out.shape) != (cols, rows):
        raise ValueError("shape mismatch")
    return Prepared("mtnn_transpose", (_stream(stream), rows, cols, pi, ldi, po, ldo), (X, out))


# ---- selection ----------------------------------------------------------------------------

def mtnn_select(m: int, n: int, k: int) -> int:
    return int(lib().mtnn_select(m, n, k))


def mtnn_select_batch(shapes):
    """Labels for many (m, n, k) at once (one library call)."""
    import numpy as np
    mnk = np.ascontiguousarray(shapes, dtype=np.int32).reshape(-1, 3)
    out = np.empty(mnk.shape[0], dtype=np.int32)
    _check(lib().mtnn_select_batch(mnk.shape[0], mnk.ctypes.data, out.ctypes.data), "mtnn_select_batch")
    return out


def mtnn_features(m: int, n: int, k: int):
    x = (ctypes.c_double * lib().mtnn_num_features())()
    _check(lib().mtnn_features(m, n, k, x), "mtnn_features")
    return list(x)


def mtnn_load_model(path: str) -> None:
    _check(lib().mtnn_load_model(os.fsencode(path)), "mtnn_load_model")


def mtnn_save_model(path: str) -> None:
    _check(lib().mtnn_save_model(os.fsencode(path)), "mtnn_save_model")


def mtnn_unload_model() -> None:
    lib().mtnn_unload_model()


def mtnn_gbdt_train(X, labels, num_trees=8, max_depth=8, eta=1.0, gamma=0.0, lam=1.0, min_child_weight=1.0):
    import numpy as np
    X = np.ascontiguousarray(X, dtype=np.float64)
    y = np.ascontiguousarray(labels, dtype=np.int32)
    _check(lib().mtnn_gbdt_train(X.shape[0], X.shape[1], X.ctypes.data, y.ctypes.data, num_trees, max_depth,
                                 eta, gamma, lam, min_child_weight), "mtnn_gbdt_train")


def mtnn_train_selector(shapes, labels) -> None:
    import numpy as np
    mnk = np.ascontiguousarray(shapes, dtype=np.int32).reshape(-1, 3)
    y = np.ascontiguousarray(labels, dtype=np.int32)
    _check(lib().mtnn_train_selector(mnk.shape[0], mnk.ctypes.data, y.ctypes.data), "mtnn_train_selector")


def model_trees():
    """The current predictor as lists of (feature, threshold, left, right, value) per tree."""
    L = lib()
    out = []
    for t in range(L.mtnn_model_num_trees()):
        rows = []
        for i in range(L.mtnn_model_tree_size(t)):
            f, l, r = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
            thr, val = ctypes.c_double(), ctypes.c_double()
            _check(L.mtnn_model_node(t, i, ctypes.byref(f), ctypes.byref(thr), ctypes.byref(l), ctypes.byref(r),
                                     ctypes.byref(val)), "mtnn_model_node")
            rows.append((f.value, thr.value, l.value, r.value, val.value))
        out.append(rows)
    return out


def mtnn_model_margin(x) -> float:
    import numpy as np
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = ctypes.c_double()
    _check(lib().mtnn_model_margin(x.ctypes.data, x.size, ctypes.byref(out)), "mtnn_model_margin")
    return out.value


def gemm_configs():
    L = lib()
    return [L.mtnn_gemm_config_name(i).decode() for i in range(L.mtnn_gemm_config_count())]


def mtnn_gemm_default_config(op: int, m: int, n: int, k: int) -> int:
    return int(lib().mtnn_gemm_default_config(op, m, n, k))


# ---- fully connected training step -------------------------------------------------------

def mtnn_fc_workspace_bytes(dims, batch: int) -> int:
    arr = (ctypes.c_int * len(dims))(*dims)
    return int(lib().mtnn_fc_workspace_bytes(len(dims) - 1, arr, batch))


def make_fc_desc(dims, batch, X, labels, W, b, dW, db, loss, workspace, lr, forward_mode=0, logits=None):
    """Fill a mtnn_fc_step_desc from device tensors.  Returns (desc, keepalive)."""
    L = len(dims) - 1
    dims_arr = (ctypes.c_int * (L + 1))(*dims)

    def ptrs(ts):
        return (_c_vp * L)(*[t.data_ptr() for t in ts])

    pw, pb, pdw, pdb = ptrs(W), ptrs(b), ptrs(dW), ptrs(db)
    desc = FcStepDesc(L, dims_arr, batch, X.data_ptr(), labels.data_ptr(), pw, pb, pdw, pdb,
                      logits.data_ptr() if logits is not None else None, loss.data_ptr(),
                      workspace.data_ptr(), workspace.numel() * workspace.element_size(), lr, forward_mode)
    return desc, (dims_arr, pw, pb, pdw, pdb)


def mtnn_fc_train_step(desc, stream=None) -> None:
    _check(lib().mtnn_fc_train_step(_stream(stream), ctypes.byref(desc)), "mtnn_fc_train_step")


def mtnn_fc_forward(desc, stream=None) -> None:
    _check(lib().mtnn_fc_forward(_stream(stream), ctypes.byref(desc)), "mtnn_fc_forward")


def mtnn_fc_bias_act(Z, b, relu: bool, stream=None):
    _check(lib().mtnn_fc_bias_act(_stream(stream), Z.shape[0], Z.shape[1], Z.data_ptr(), b.data_ptr(), int(relu)),
           "mtnn_fc_bias_act")


def mtnn_fc_softmax_xent(logits, labels, dZ, row_loss, mean_loss, stream=None):
    _check(lib().mtnn_fc_softmax_xent(_stream(stream), logits.shape[0], logits.shape[1], logits.data_ptr(),
                                      labels.data_ptr(), dZ.data_ptr(), row_loss.data_ptr(), mean_loss.data_ptr()),
           "mtnn_fc_softmax_xent")


def mtnn_fc_relu_backward(dH, H, stream=None):
    _check(lib().mtnn_fc_relu_backward(_stream(stream), dH.numel(), dH.data_ptr(), H.data_ptr()),
           "mtnn_fc_relu_backward")


def mtnn_fc_bias_grad(dZ, db, scratch=None, stream=None):
    _check(lib().mtnn_fc_bias_grad(_stream(stream), dZ.shape[0], dZ.shape[1], dZ.data_ptr(), db.data_ptr(),
                                   scratch.data_ptr() if scratch is not None else None), "mtnn_fc_bias_grad")


def mtnn_fc_relu_backward_bias_grad(dH, H, db, scratch=None, stream=None):
    """dH <- where(H > 0, dH, 0) in place and db <- column sums of the result, in one pass."""
    _check(lib().mtnn_fc_relu_backward_bias_grad(_stream(stream), dH.shape[0], dH.shape[1], dH.data_ptr(), H.data_ptr(),
                                                 db.data_ptr(), scratch.data_ptr() if scratch is not None else None),
           "mtnn_fc_relu_backward_bias_grad")


def mtnn_fc_sgd(P, G, lr: float, stream=None):
    _check(lib().mtnn_fc_sgd(_stream(stream), P.numel(), P.data_ptr(), G.data_ptr(), lr), "mtnn_fc_sgd")


def mtnn_fc_layer_forward(X, W, b, Y, relu: bool, mode: int = 0, workspace=None, stream=None) -> int:
    """Y = act(X x W^T + b) with the bias and the clamp in the product's epilogue.  mode: +1 NT, -1 TNN,
    0 the predictor's choice; returns the path that ran (+1 / -1)."""
    (px, ldx), (pw_, ldw), (py, ldy) = _dev(X, "X"), _dev(W, "W"), _dev(Y, "Y")
    m, k = X.shape
    n = W.shape[0]
    pw, wb = _ws(workspace)
    chosen = ctypes.c_int(0)
    _check(lib().mtnn_fc_layer_forward(_stream(stream), mode, m, n, k, px, ldx, pw_, ldw, b.data_ptr(), 1 if relu else 0,
                                       py, ldy, pw, wb, ctypes.byref(chosen)), "mtnn_fc_layer_forward")
    return chosen.value


def mtnn_fc_weight_grad_sgd(A, B, dW, W, lr: float, stream=None):
    """dW = A x B (NN) and W = fma(-lr, dW, W), the update in the product's epilogue."""
    (pa, lda), (pb, ldb), (pg, ldg), (pw_, ldw) = _dev(A, "A"), _dev(B, "B"), _dev(dW, "dW"), _dev(W, "W")
    m, k = A.shape
    n = B.shape[1]
    _check(lib().mtnn_fc_weight_grad_sgd(_stream(stream), m, n, k, pa, lda, pb, ldb, pg, ldg, pw_, ldw, lr),
           "mtnn_fc_weight_grad_sgd")
    return dW


def mtnn_copy_bytes(src, dst, stream=None):
    """Streaming device copy of a whole tensor (the known-traffic calibration kernel)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("size mismatch")
    _check(lib().mtnn_copy_bytes(_stream(stream), nbytes, src.data_ptr(), dst.data_ptr()), "mtnn_copy_bytes")
    return dst


def mtnn_probe_lanes(n_mfma: int, n_valu: int, sink, stream=None):
    """The overlap probe of csrc/probe.hip: n_mfma matrix instructions and n_valu vector multiply-adds per SIMD."""
    _check(lib().mtnn_probe_lanes(_handle(stream) or None, n_mfma, n_valu, sink.data_ptr()), "mtnn_probe_lanes")


def mtnn_gemm_default_splits(op: int, m: int, n: int, k: int) -> int:
    return int(lib().mtnn_gemm_default_splits(op, m, n, k))


def mtnn_gemm_scratch_bytes(cfg: int, splits: int, m: int, n: int, k: int) -> int:
    """Scratch a (cfg, splits) launch needs for its partial products; 0 for an unsplit launch."""
    return int(lib().mtnn_gemm_scratch_bytes(cfg, splits, m, n, k))


def mtnn_gemm_choice(op: int, m: int, n: int, k: int, scratch_bytes: Optional[int] = None):
    """(cfg, splits) the cost model picks for aligned operands with that much scratch (default: the default capacity)."""
    if scratch_bytes is None:
        scratch_bytes = int(lib().mtnn_scratch_bytes_default())
    c, s = ctypes.c_int(), ctypes.c_int()
    _check(lib().mtnn_gemm_choice(op, m, n, k, scratch_bytes, ctypes.byref(c), ctypes.byref(s)), "mtnn_gemm_choice")
    return c.value, s.value


def mtnn_get_scratch_bytes(stream=None) -> int:
    return int(lib().mtnn_get_scratch_bytes(_handle(stream) or None))


def mtnn_status_string(status: int) -> str:
    return lib().mtnn_status_string(status).decode()


EVEN_CUT = -2      # `splits` value of mtnn_gemm_ex: cut all tiles' k ranges evenly over a fixed grid


def mtnn_gemm_even_cut_launches() -> int:
    return int(lib().mtnn_gemm_even_cut_launches())


def mtnn_gemm_fused_epilogue_launches() -> int:
    return int(lib().mtnn_gemm_fused_epilogue_launches())


def mtnn_set_fused_epilogues(enable: bool) -> bool:
    """Process-wide switch for measurements: False = separate bias / ReLU / SGD passes.  Returns the old setting."""
    return bool(lib().mtnn_set_fused_epilogues(1 if enable else 0))


def mtnn_device_attribute(what: int) -> int:
    """0 compute units, 1 peak shader clock (kHz), 2 peak memory clock (kHz), 3 memory bus width (bits); -1 if unknown."""
    return int(lib().mtnn_device_attribute(what))


def mtnn_version() -> int:
    return int(lib().mtnn_version())
