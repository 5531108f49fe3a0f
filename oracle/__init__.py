"""CPU oracle: the plain definitions the HIP path is checked against.

TEST INFRASTRUCTURE ONLY.  Nothing here is part of the product: only the tests,
the smoke check and the benchmark's cpu_baseline leg may import it, and it
imports nothing from the product package.  The arithmetic lives in
``mtnn_oracle.c`` (dense operations), ``selection.py`` (label rule, metrics,
boosted trees) and ``fc.py`` (one training step of a fully connected net).
"""
from .gemm import nt_ref, nn_ref, transpose_ref, tnn_ref, num_threads, nt_f64, nn_f64, tn_f64  # noqa: F401
