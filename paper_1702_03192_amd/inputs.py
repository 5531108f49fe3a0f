"""Seeded synthetic inputs shared by the tests, the bench and the smoke check.

This module only draws numbers.  It holds none of the method's arithmetic (no
product, transpose, label rule or tree code), so both the CPU oracle's tests and
the HIP path's tests may take their operands from it without sharing anything
that could hide a mistake.

Every element is a pure function of ``(seed, matrix_id, i, j)``: a 64-bit
counter is pushed through a fixed avalanche mixer, so any element of any matrix
can be regenerated alone, whatever the matrix size.  The workloads follow the
paper's experiments, which are synthetic shapes themselves (Section IV-A data
collection: only m, n, k matter) and fully connected layers described by their
sizes (Table IX).
"""
from __future__ import annotations

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix64(x: np.ndarray) -> np.ndarray:
    """Avalanche a uint64 array (xor-shift / multiply rounds); wraps modulo 2**64."""
    x = x.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        x += np.uint64(0x9E3779B97F4A7C15)
        x ^= x >> np.uint64(30)
        x *= np.uint64(0xBF58476D1CE4E5B9)
        x ^= x >> np.uint64(27)
        x *= np.uint64(0x94D049BB133111EB)
        x ^= x >> np.uint64(31)
    return x


def _bits(seed: int, matrix_id: int, rows: int, cols: int, stream: int = 0) -> np.ndarray:
    """uint64 random bits for every (i, j) of a rows x cols matrix."""
    key = _mix64(np.array([(seed & 0xFFFFFFFF) | ((matrix_id & 0xFFFF) << 32) | ((stream & 0xFFFF) << 48)],
                          dtype=np.uint64))[0]
    i = np.arange(rows, dtype=np.uint64).reshape(-1, 1)
    j = np.arange(cols, dtype=np.uint64).reshape(1, -1)
    with np.errstate(over="ignore"):
        ctr = (i << np.uint64(32)) | j
        return _mix64(ctr ^ key)


def uniform_pm1(seed: int, matrix_id: int, rows: int, cols: int) -> np.ndarray:
    """float32 matrix, i.i.d. uniform on [-1, 1): 24 random bits scaled, exact in fp32."""
    b = _bits(seed, matrix_id, rows, cols)
    u24 = (b >> np.uint64(40)).astype(np.float64)          # 0 .. 2**24-1
    return (u24 * (2.0 ** -23) - 1.0).astype(np.float32)


def normal01(seed: int, matrix_id: int, rows: int, cols: int) -> np.ndarray:
    """float32 matrix, i.i.d. N(0, 1) by the Box-Muller transform of two counter streams."""
    b1 = _bits(seed, matrix_id, rows, cols, stream=1)
    b2 = _bits(seed, matrix_id, rows, cols, stream=2)
    u1 = ((b1 >> np.uint64(11)).astype(np.float64) + 1.0) * (2.0 ** -53)   # (0, 1]
    u2 = (b2 >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)           # [0, 1)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return z.astype(np.float32)


def small_integers(seed: int, matrix_id: int, rows: int, cols: int, lo: int = -8, hi: int = 8) -> np.ndarray:
    """float32 matrix of integers drawn uniformly from [lo, hi]; sums of products stay exact in fp32."""
    b = _bits(seed, matrix_id, rows, cols, stream=3)
    span = np.uint64(hi - lo + 1)
    return ((b >> np.uint64(33)) % span).astype(np.int64).__add__(lo).astype(np.float32)


def index_coded(rows: int, cols: int) -> np.ndarray:
    """float32 matrix with X[r][c] = r * 4096 + c: every entry distinct and exact (rows, cols <= 4096)."""
    if rows > 4096 or cols > 4096:
        raise ValueError("index_coded is exact in fp32 only up to 4096 x 4096")
    r = np.arange(rows, dtype=np.float32).reshape(-1, 1)
    c = np.arange(cols, dtype=np.float32).reshape(1, -1)
    return r * np.float32(4096.0) + c


def uniform_ints(seed: int, stream_id: int, count: int, lo: int, hi: int) -> np.ndarray:
    """int64 vector of `count` integers uniform on [lo, hi] (class labels, random shapes)."""
    b = _bits(seed, stream_id, 1, count, stream=4)[0]
    return ((b >> np.uint64(20)) % np.uint64(hi - lo + 1)).astype(np.int64) + lo


def xavier_uniform(seed: int, matrix_id: int, fan_out: int, fan_in: int) -> np.ndarray:
    """float32 weight matrix W[fan_out][fan_in], uniform on [-b, b), b = sqrt(6 / (fan_in + fan_out))."""
    bound = np.float64(np.sqrt(6.0 / (fan_in + fan_out)))
    return (uniform_pm1(seed, matrix_id, fan_out, fan_in).astype(np.float64) * bound).astype(np.float32)


def with_leading_dim(x: np.ndarray, ld: int, fill: float = np.nan) -> np.ndarray:
    """Copy x (rows x cols) into a rows x ld buffer whose padding columns hold `fill`."""
    rows, cols = x.shape
    if ld < cols:
        raise ValueError("ld must be >= cols")
    buf = np.full((rows, ld), fill, dtype=x.dtype)
    buf[:, :cols] = x
    return buf


# --- the workloads of the benchmark configurations -------------------------------------------

SWEEP_SIZES = (64, 128, 256, 512, 1024, 2048, 4096, 8192)

CONFIG1 = {"name": "single_nt_256", "shapes": [(256, 256, 256)], "dist": "uniform", "seeds": [1702]}
CONFIG2 = {"name": "fc_layer_nt", "shapes": [(1024, 4096, 4096), (4096, 4096, 1024)], "dist": "uniform",
           "seeds": [3192, 3193]}
CONFIG4 = {"name": "skinny_irregular", "dist": "normal",
           "shapes": [(32, 8192, 8192), (8192, 32, 8192), (8192, 8192, 32), (1000, 1000, 1000), (3000, 1500, 4500)],
           "seeds": [4000, 4001, 4002, 4003, 4004]}
CONFIG5 = {"name": "fc_step", "dims": [784, 4096, 4096, 4096, 10], "batch": 1024, "seed": 5000}


def sweep_shapes():
    """The 512 (m, n, k) of the selector sweep, with the per-shape seed."""
    out = []
    for im, m in enumerate(SWEEP_SIZES):
        for in_, n in enumerate(SWEEP_SIZES):
            for ik, k in enumerate(SWEEP_SIZES):
                out.append((m, n, k, 10000 + 64 * im + 8 * in_ + ik))
    return out


def nt_operands(m: int, n: int, k: int, seed: int, dist: str = "uniform"):
    """A (m x k) and B (n x k) for one NT operation."""
    gen = {"uniform": uniform_pm1, "normal": normal01, "int": small_integers}[dist]
    return gen(seed, 0, m, k), gen(seed, 1, n, k)
