"""MI355X-native TurboRAG online-prefill hot path (arXiv 2410.07590).

The product is the C-ABI library built from csrc/ (declared in include/turborag.h);
`binding` is a thin ctypes layer over it with the same names.  Nothing is imported
eagerly so that the seeded input generators (`synth`) and the work accounting
(`accounting`) can be used without the HIP library present.
"""
__all__ = ["binding", "synth", "accounting", "build"]
