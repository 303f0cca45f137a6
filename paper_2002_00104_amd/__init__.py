"""PWLQ breakpoint search + quantizer for MI355X (gfx950).

``paper_2002_00104_amd.pwlq`` is the ctypes binding over the C-ABI library
``libpwlq.so`` (hand-written HIP).  ``paper_2002_00104_amd.synth`` holds the
seeded input generators.  Nothing is imported eagerly so that the input
generators can be used without the GPU library being built.
"""

__all__ = ["pwlq", "synth"]
