"""MI355X-native fused sliding-window + residual-linear attention (RAttention layer).

The compute lives in librattn.so (hand-written HIP for gfx950) behind a C ABI declared in
include/rattn.h; `binding` marshals torch device tensors into it.  Importing the package
does not load the library; `binding.lib()` does and raises if it is not built.
"""
__all__ = ["binding", "synth", "build"]
