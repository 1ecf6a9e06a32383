"""MI355X-native change-based convolution (CBinfer, arXiv 1704.04313): thin Python binding
over the C ABI of libcbinfer_hip.so.  All computation runs in the HIP kernels; this package
only marshals arguments."""
from .binding import (CBInfer, CBInferError, library_path, load_library, LIST_CHANGED, LIST_UPDATE, LIST_POOLED,
                      MAP_REFERENCE, MAP_OUTPUT, STEP_NAMES, FLAG_HOLD_REFERENCE, FLAG_LISTS_EVERY_FRAME, FLAG_PIPELINE_FRAMES, OP_CONV, OP_MAXPOOL,
                      cbinfer_workspace_bytes, F32, BF16)

__all__ = ["CBInfer", "CBInferError", "library_path", "load_library", "LIST_CHANGED", "LIST_UPDATE", "LIST_POOLED",
           "MAP_REFERENCE", "MAP_OUTPUT", "STEP_NAMES", "FLAG_HOLD_REFERENCE", "FLAG_LISTS_EVERY_FRAME", "FLAG_PIPELINE_FRAMES", "OP_CONV", "OP_MAXPOOL",
           "cbinfer_workspace_bytes", "F32", "BF16"]
