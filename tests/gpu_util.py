"""Helpers for the GPU parity tests: device buffers with guard bands, tolerance checks."""
import numpy as np

CANARY_BITS = 0x7FC0DEAD          # a quiet NaN with a recognisable payload


def tol(k):
    """GEMM tolerance of the benchmark definition: max relative error <= 1e-5 * sqrt(k)."""
    return 1e-5 * np.sqrt(max(k, 1))


def dev_matrix(x, ld=None, fill=np.nan, misalign=0):
    """Upload a host matrix into a device buffer with leading dimension ld (padding = fill).
    `misalign` shifts the base by that many words off the allocation's 16-byte alignment.
    Returns the rows x cols device view."""
    import torch
    rows, cols = x.shape
    ld = cols if ld is None else ld
    flat = np.full(misalign + rows * ld, fill, dtype=np.float32)
    body = flat[misalign:].reshape(rows, ld)
    body[:, :cols] = x
    t = torch.from_numpy(flat).cuda()
    return t[misalign:].view(rows, ld)[:, :cols]


class Guarded:
    """A rows x cols fp32 device output inside a canary-filled buffer: `guard` words before and
    after, and ld - cols padding words per row.  check() verifies no canary was overwritten."""

    def __init__(self, rows, cols, ld=None, guard=1024, misalign=0):
        import torch
        self.rows, self.cols = rows, cols
        self.ld = cols if ld is None else ld
        self.guard = guard + misalign
        total = self.guard + rows * self.ld + guard
        host = np.full(total, CANARY_BITS, dtype=np.uint32)
        self.flat = torch.from_numpy(host.view(np.int32)).cuda()
        body = self.flat[self.guard:self.guard + rows * self.ld].view(torch.float32)
        self.view = body.view(rows, self.ld)[:, :cols] if rows and self.ld else body.view(rows, cols)

    def host(self):
        """(matrix, intact): the logical matrix as fp32 numpy, and whether all canaries survive."""
        raw = self.flat.cpu().numpy().view(np.uint32)
        g, r, ld, c = self.guard, self.rows, self.ld, self.cols
        intact = bool(np.all(raw[:g] == CANARY_BITS) and np.all(raw[g + r * ld:] == CANARY_BITS))
        body = raw[g:g + r * ld].reshape(r, ld) if r and ld else raw[g:g].reshape(r, max(ld, 1))
        if ld > c and r:
            intact = intact and bool(np.all(body[:, c:] == CANARY_BITS))
        return body[:, :c].copy().view(np.float32), intact


def check_gemm(C_gpu, C_ref, S_ref, k, what=""):
    """Both readings of 'max relative error <= 1e-5 sqrt(k)': componentwise against
    S = |A||B| and normwise against max|C|.  Returns the two measured errors."""
    C_gpu = np.asarray(C_gpu, dtype=np.float64)
    assert C_gpu.shape == C_ref.shape, what
    assert np.isfinite(C_gpu).all(), f"{what}: non-finite output"
    diff = np.abs(C_gpu - C_ref)
    denom = np.where(S_ref > 0, S_ref, 1.0)
    comp = float((diff / denom).max()) if diff.size else 0.0
    norm = float(diff.max() / max(np.abs(C_ref).max(), 1e-300)) if diff.size else 0.0
    assert comp <= tol(k), f"{what}: componentwise error {comp:.3e} > {tol(k):.3e}"
    assert norm <= tol(k), f"{what}: normwise error {norm:.3e} > {tol(k):.3e}"
    return comp, norm


def check_gemm_on_device(C_dev, C_ref, S_ref, k, what=""):
    """check_gemm for large results: the same two readings of the tolerance, with the elementwise
    comparison arithmetic (subtract, divide, max -- nothing of the method) done by torch in float64 on
    the device instead of numpy on the host.  C_dev: fp32 device tensor; C_ref, S_ref: the oracle's
    float64 host arrays."""
    import torch
    assert tuple(C_dev.shape) == C_ref.shape, what
    got = C_dev.double()
    assert bool(torch.isfinite(got).all()), f"{what}: non-finite output"
    ref = torch.from_numpy(np.ascontiguousarray(C_ref)).cuda()
    s = torch.from_numpy(np.ascontiguousarray(S_ref)).cuda()
    diff = (got - ref).abs_()
    norm = float(diff.max() / ref.abs().max().clamp_min(1e-300)) if diff.numel() else 0.0
    comp = float((diff / torch.where(s > 0, s, torch.ones_like(s))).max()) if diff.numel() else 0.0
    assert comp <= tol(k), f"{what}: componentwise error {comp:.3e} > {tol(k):.3e}"
    assert norm <= tol(k), f"{what}: normwise error {norm:.3e} > {tol(k):.3e}"
    return comp, norm
