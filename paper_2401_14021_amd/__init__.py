"""MI355X-native hot path of RaLMSpec: exact dense retrieval (batched
maximum-inner-product top-k), the per-request speculation-cache top-1 lookup
and the batched-verification first-mismatch compare (Alg. 1 of the paper).

The compute lives in ``libralm.so`` (hand-written HIP for gfx950, C ABI declared
in ``include/ralm.h``).  ``paper_2401_14021_amd.binding`` marshals torch
tensors onto that ABI; ``paper_2401_14021_amd.inputs`` holds the seeded
synthetic input generators.  Nothing is loaded at import time, so the input
generators can be used on a machine without a GPU.
"""

__all__ = ["binding", "inputs", "build"]
