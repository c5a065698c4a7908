"""MI355X-native PeRQ online activation path: permute -> block Hadamard -> INT4 / MXFP4.

`binding` loads the C-ABI library (libperq.so, built by `build.build()`); `synth` holds the
seeded input generators.  Nothing is loaded at import time.
"""
__all__ = ["binding", "build", "synth"]
