"""MI355X-native local-block training step of PPLL (hand-written HIP behind a C ABI).

`binding` marshals arguments for libppll.so; `synth` generates seeded workloads.
The shared library is loaded on first use and its absence is an error: there is
no CPU fallback.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
