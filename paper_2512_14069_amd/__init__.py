"""MI355X-native hot path of RADAR's speculative-sampling loop (arXiv 2512.14069).

The work is done by hand-written HIP kernels in libradar.so (C ABI in
include/radar.h); ``binding`` marshals torch GPU tensors into those calls and
``synth`` makes the seeded synthetic inputs.  Attributes of ``binding`` are
re-exported lazily so that importing the package (or ``synth``) needs neither
torch nor the built library.
"""
import importlib

__all__ = ["binding", "synth", "build"]


def __getattr__(name):
    if name in ("binding", "synth", "build"):
        return importlib.import_module(f"{__name__}.{name}")
    binding = importlib.import_module(f"{__name__}.binding")
    if hasattr(binding, name):
        return getattr(binding, name)
    raise AttributeError(name)
