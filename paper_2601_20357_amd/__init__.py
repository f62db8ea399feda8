"""TABED per-round hot path for MI355X (gfx950): HIP kernels behind a C-ABI.

`binding` wraps libtabed.so (argument marshalling only); `synth` draws the
seeded synthetic inputs.  Importing this package touches neither the GPU nor
the shared library; `binding.load()` fails loudly if the library is missing.
"""
__all__ = ["binding", "synth", "build"]
