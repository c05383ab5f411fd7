"""MI355X-native forward convolution layer (conv + bias + fused ReLU, fp32).

The arithmetic lives in hand-written HIP kernels for gfx950 behind the C ABI
declared in ``include/bconv.h`` (built into ``libbconv.so`` next to this file);
``binding`` marshals torch device pointers into it.  Nothing here falls back to
the CPU: if the library is missing, calls raise.
"""
__all__ = ["binding", "roofline", "build"]
