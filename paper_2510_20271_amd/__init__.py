"""MI355X-native Euler Characteristic Curves (hard and soft) behind a C ABI.

``api`` binds the entry points of include/ecc.h; ``synth`` holds the seeded
synthetic inputs; ``build`` compiles the HIP sources for gfx950.
"""
__all__ = ["api", "synth", "build"]
