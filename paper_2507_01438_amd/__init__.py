"""MI355X-native batched multi-adapter LoRA linear layer (batch LoRA inference, Sec. 3.4 of the paper).

Sub-modules:
  inputs   seeded synthetic workloads (no layer arithmetic; imports nothing from the HIP path)
  binding  ctypes binding of libelora.so (the C-ABI declared in include/elora.h); importing it
           fails loudly if the HIP library has not been built
"""

__all__ = ["inputs", "binding"]
