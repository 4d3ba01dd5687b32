"""MI355X-native CAOTE hot path: score, select and compact cached KV tokens.

The work is done by hand-written HIP kernels for gfx950 behind a C ABI
(``include/caote.h``, built to ``libcaote_hip.so``); ``binding`` only marshals
arguments.  ``synth`` holds the seeded input generators.  There is no CPU
fallback: calling an entry point without the built library raises.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
