"""MI355X-native Euler Characteristic Curves (hard and soft) behind a C ABI.

``api`` binds the entry points of include/ecc.h; ``layer`` wraps the soft path as a
``torch.autograd.Function`` / ``nn.Module``; ``synth`` holds the seeded synthetic
inputs; ``build`` compiles the HIP sources for gfx950.
"""
__all__ = ["api", "layer", "synth", "build"]
