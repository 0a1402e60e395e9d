"""MI355X-native kernels for the co-serving attention / KV-cache hot path.

Four per-layer device operations behind a C ABI (``include/conserve_kv.h``), hand-written
HIP for gfx950: append of a step's new K/V into 16-token pages, paged attention over a
mixed batch of decode tokens and chunked-prefill tokens, and the checkpoint gather /
restore copies of incremental KV checkpointing.

``paper_2410_01228_amd.binding`` -- ctypes binding with the C names (loads the built
                                    library, raises if it is missing).
``paper_2410_01228_amd.synth``   -- seeded synthetic workloads (no arithmetic of the method).
"""

__all__ = ["binding", "synth"]
