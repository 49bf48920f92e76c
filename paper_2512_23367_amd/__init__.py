"""MI355X (gfx950) quantized linear layer: W8A8 / W4A8 GEMMs behind a C-ABI library.

`paper_2512_23367_amd.binding` wraps the C entry points declared in
include/qlinear.h (loaded lazily; a missing library is an error, there is no
fallback).  `paper_2512_23367_amd.synth` draws the seeded synthetic inputs.
"""
__all__ = ["binding", "synth", "build"]
