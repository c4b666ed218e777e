"""MI355X-native decode-step hot path of ESS (arXiv 2512.10576).

`paper_2512_10576_amd.binding` is the thin ctypes layer over the C-ABI
library `libess.so` (built from `csrc/` for gfx950); `synth` draws seeded
synthetic inputs.  Importing the package does not load the library;
`binding.load()` does, and raises if it has not been built.
"""
__all__ = ["binding", "synth", "build"]
