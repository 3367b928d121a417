"""MI355X-native W4A4 static-quantized linear layer (FPTQuant inference hot path).

`binding` holds the ctypes view of the C-ABI library built from csrc/.  Nothing here falls back to
a CPU implementation: without the HIP library the calls raise.
"""
__all__ = ["binding", "build"]
