"""MI355X-native inference of the lightweight student Transformer (arXiv 2109.08003).

Thin ctypes binding over libnt.so; every numerical step runs in the library's gfx950 kernels.
"""
from .binding import (NtError, Model, lib, load_library, n_steps, param_count, plan_batches,  # noqa: F401
                      EXPORTS, make_config, kernel_names, q8_quantize_row)
