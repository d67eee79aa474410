"""MI355X-native worker hot path of the RoundPipe schedule: a C-ABI HIP library (librp.so) and its ctypes binding.

`binding` mirrors include/rp.h and include/rp_ops.h one to one; `harness` packs weights and owns torch buffers.
Importing `binding` without a built library raises: there is no CPU fallback.
"""
