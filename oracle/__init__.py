"""CPU oracle for the chunk-backed decode-attention path. TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package; the GPU
library and its Python binding never do.
"""
from .model import OraclePool, OracleError, load  # noqa: F401
