"""Clustered, compressed MoE FFN layer forward for MI355X: thin binding over libcmoe.so.

All compute runs in the HIP library (include/cmoe.h); this package only marshals
arguments.  PyTorch supplies device memory and streams.
"""
from .binding import (CmoeError, Layer, calibrate_mfma, compress, lib, lib_path, quantize_int4,  # noqa: F401
                      reconstruction_error, status_string)
