"""MI355X-native stage-compute hot path (HIP kernels behind the C ABI of include/dpipe.h).

The Python layer only marshals arguments; every step runs in libdpipe.so.
Importing the package does not load the library; the first call does, and it
raises if the library has not been built (no CPU fallback exists).
"""
from .binding import (DP_BF16, DP_F32, KIND_DIT, KIND_UNET, DpipeError, Encoder, ImageEncoder, LayerCost, Stage, library_path, load_library)

__all__ = ["DP_BF16", "DP_F32", "KIND_DIT", "KIND_UNET", "DpipeError", "Encoder", "ImageEncoder", "LayerCost", "Stage", "library_path",
           "load_library"]
