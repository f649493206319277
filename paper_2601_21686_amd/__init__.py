"""MI355X-native decode attention over a low-rank projected KV cache.

`paper_2601_21686_amd.binding` wraps the C-ABI library (include/skv.h);
`paper_2601_21686_amd.synth` holds the seeded input generators;
`paper_2601_21686_amd.build` compiles the HIP sources for gfx950.
Nothing is loaded at import time: the shared library is opened on first use
and a missing library is an error, never a fallback.
"""
__all__ = ["binding", "synth", "build"]
