"""MI355X-native fused dequantize-and-multiply for Inferflow's block-quantized weights.

`paper_2401_08294_amd.iflow` is the thin ctypes binding over the C-ABI library `libiflow.so`
(declared in `include/iflow.h`); `paper_2401_08294_amd.synth` draws seeded synthetic inputs.
Importing the package does not load the GPU library; `iflow.lib()` does, and fails loudly when the
library has not been built.
"""
__all__ = ["iflow", "synth", "build"]
