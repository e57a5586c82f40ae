"""MI355X-native hybrid dense / 2:4 tile linear layer (the inference path of PATCH, arXiv 2509.23410).

The compute lives in a C-ABI shared library built from ``csrc/`` (hand-written HIP for gfx950);
``binding`` is a thin ctypes layer over it and ``synth`` draws seeded synthetic inputs.  Nothing is
loaded at import time; the first call into ``binding`` loads the library and fails loudly if it is
missing.
"""
__all__ = ["binding", "synth"]
