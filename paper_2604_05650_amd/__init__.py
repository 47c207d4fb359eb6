"""MI355X-native verify-step hot path of LVSpec (loosely speculative decoding for Video-LLMs).

``paper_2604_05650_amd.binding`` is the thin ctypes layer over the C-ABI library
``liblvspec.so`` (hand-written HIP kernels for gfx950); ``paper_2604_05650_amd.synth`` holds the
seeded synthetic-input generators and nothing of the method's arithmetic.  Attribute access is
lazy so that importing the generators never loads the GPU library.
"""
import importlib

__all__ = ["binding", "synth", "build"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
