"""MI355X-native dual-mode W4 linear layer of QSpec (arXiv 2410.11305).

`binding` exposes the C ABI of libqspec.so (hand-written HIP for gfx950);
`synth` draws the seeded benchmark inputs; `build` compiles the library."""
from . import synth  # noqa: F401

__all__ = ["binding", "synth", "build"]
