"""MI355X (gfx950) Winograd 3x3 convolution: thin Python binding over libwino.so.

Importing this package loads nothing native; the library is opened on the first
call into ``paper_2412_05781_amd.binding`` and that fails loudly if it has not
been built (there is no CPU fallback).
"""
__all__ = ["binding", "synth", "build"]
