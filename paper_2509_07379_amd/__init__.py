"""MI355X-native MoE FFN layer served from an offloaded expert pool.

`paper_2509_07379_amd.binding` is the thin ctypes layer over the C-ABI library
(libmoe_offload.so, built from csrc/ with hipcc for gfx950); it raises if the
library is missing.  `paper_2509_07379_amd.synth` holds the seeded input generators.
"""
__all__ = ["binding", "synth"]
