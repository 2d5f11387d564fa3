"""MI355X-native module-replica hot path (CoCoServe's replicate / forward-split / migrate).

Python side = argument marshalling over the C ABI declared in include/cocoserve_mi.h; every
step of the path runs in the HIP kernels of libcocoserve_mi.so.  There is no CPU fallback:
importing `binding` fails loudly when the library has not been built.
"""
from .binding import (  # noqa: F401
    CCS_BF16, CCS_DECODE, CCS_DECODER_LAYER, CCS_F32, CCS_LINEAR, CCS_PREFILL, CCS_ROWS,
    CcsError, Module, ModuleDesc, lib, lib_path,
)
