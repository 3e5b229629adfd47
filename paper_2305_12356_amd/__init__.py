"""MI355X (gfx950) library for the quantize-and-score / format-select hot path of
Mixture-of-Formats Quantization (arXiv 2305.12356).

`binding` wraps the C ABI declared in include/mofq.h (libmofq.so, built from
csrc/*.hip by `build`).  Importing `binding` raises if the library is not built:
there is no fallback implementation.
"""
__all__ = ["binding", "build"]
