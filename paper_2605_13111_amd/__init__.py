"""Ragged-cache attention for Pyramid Forcing on MI355X (gfx950).

``paper_2605_13111_amd.binding`` wraps the C ABI declared in ``include/pf.h``
(``libpf.so``, hand-written HIP); ``paper_2605_13111_amd.synth`` holds the seeded
synthetic workloads.  The binding is imported lazily so that the input module
can be used on machines without the built library.
"""

__all__ = ["synth", "binding"]
