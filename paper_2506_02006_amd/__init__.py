"""MI355X-native fp16 / W4A16 linear layers for mixed-precision (layer-swapped) serving.

The compute lives in csrc/ (HIP, gfx950) behind the C ABI declared in include/morph.h;
`binding` marshals torch device pointers into that ABI.  `synth` only generates inputs.
Nothing is loaded at import time: `from paper_2506_02006_amd import binding` loads the library.
"""
__all__ = ["synth", "binding"]
