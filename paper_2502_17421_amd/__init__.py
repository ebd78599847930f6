"""MI355X-native hybrid tree attention (LongSpec, Section 3.3).

``paper_2502_17421_amd.binding`` is the thin ctypes layer over the C-ABI HIP library
(``include/ls_attn.h``); ``paper_2502_17421_amd.synth`` draws seeded synthetic inputs.
Nothing here falls back to a CPU implementation: without the built library every
call raises.
"""
__all__ = ["binding", "synth", "build"]
