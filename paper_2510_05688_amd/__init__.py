"""vAttention decode step on MI355X: thin Python face of libvatt (HIP, gfx950).

`binding` mirrors the C ABI of include/vatt.h one to one; `session.DecodeSession`
only allocates device buffers with PyTorch and hands their addresses over.
Submodules are loaded on first use so that `python -m paper_2510_05688_amd.build`
works before the library exists; `binding` raises if libvatt.so is missing.
"""
import importlib

__all__ = ["binding", "session", "build", "DecodeSession"]


def __getattr__(name):
    if name in ("binding", "session", "build"):
        return importlib.import_module("." + name, __name__)
    if name == "DecodeSession":
        return importlib.import_module(".session", __name__).DecodeSession
    raise AttributeError(name)
