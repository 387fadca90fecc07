"""MI355X-native H-BitLinear forward path (BitNet v2, Section 2.1).

``paper_2504_18415_amd.hbl`` is the thin ctypes binding over the C-ABI library
``libhbitlinear.so`` built from ``csrc/``; ``paper_2504_18415_amd.synth`` holds
the seeded synthetic-input generators.  Nothing is loaded at import time.
"""

__all__ = ["hbl", "synth"]
