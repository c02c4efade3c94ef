"""ESP decode step for MI355X (gfx950): thin Python binding over a C-ABI HIP library.

`synth` (seeded inputs) imports without the native library; everything else lives in
`binding`, which loads libesp_hip.so and fails loudly when it is missing.
"""

__all__ = ["synth", "binding"]
