"""MI355X-native per-GPU compute path of PTD-P training (arXiv 2104.04473).

The work happens in ``libptdp.so`` (hand-written HIP for gfx950, C ABI declared in
``include/ptdp.h``).  This package only marshals arguments: ``binding`` mirrors the
C entry points one to one, ``synth`` generates seeded synthetic inputs.  There is no
CPU fallback: if the library has not been built, importing ``binding`` raises.
"""
__all__ = ["binding", "synth", "build"]
