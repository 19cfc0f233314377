"""Batched Go (and Hex) environment step for AMD MI355X: thin Python binding of the C ABI in include/pgxgo.h
and include/pgxhex.h.

Argument marshalling only: every rule step runs in the HIP kernels of libpgxgo.so.  PyTorch is used
for device memory and for the HIP stream, nothing else.  There is no CPU fallback: loading fails
loudly when the library has not been built (python paper_2303_17503_amd/build.py).
"""
from .binding import GoEnv, PgxGoError, lib, lane_shift_probe, fill_probe, empty_probe, LIB_PATH  # noqa: F401
from .hex_binding import HexEnv  # noqa: F401
