"""MI355X-native LSH reduced-vocabulary softmax + beam expansion (thin binding over the C ABI).

Every step of the path runs in the HIP kernels of liblshbeam.so; this package only marshals
arguments.  PyTorch is used for device memory and streams, nothing else.  There is no CPU
fallback: if the library is missing or no GPU is present the calls raise.
"""
from .binding import (LshBeamError, Tables, build_tables, decode_step, kernel_names, load_library,
                      library_path, step_workspace_bytes)

__all__ = ["LshBeamError", "Tables", "build_tables", "decode_step", "kernel_names",
           "load_library", "library_path", "step_workspace_bytes"]
