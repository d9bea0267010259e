"""CPU oracle of the decoder -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It wraps jpeg_oracle.c (a plain sequential baseline-JPEG decoder,
double-precision pixel path) through ctypes and imports nothing from the GPU
package or from the input generators.
"""
from .oracle import (OracleError, OracleImage, build, idct8x8, idct_scaled, unstuff_bytes, zigzag)

__all__ = ["OracleError", "OracleImage", "build", "idct8x8", "idct_scaled", "unstuff_bytes", "zigzag"]
