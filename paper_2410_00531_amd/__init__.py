"""MI355X-native hot path of TPI-LLM's tensor-parallel inference: one shard's
decoder-layer forward, the fixed-order star reduce and the sliding weight
window, as hand-written HIP kernels behind a C ABI (``include/tpi.h``).

Importing the package loads nothing native; ``paper_2410_00531_amd.binding``
loads ``libtpi.so`` on first use and raises if it is missing.
"""
__all__ = ["configs", "synth"]
