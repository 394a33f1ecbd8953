"""MI355X-native Parallax attention forward (decode + prefill) behind a C ABI.

`binding` exposes the library's entry points under the names of include/parallax.h;
`synth` draws the seeded synthetic inputs of the benchmark configurations.
"""
from . import synth  # noqa: F401

__all__ = ["binding", "synth"]


def __getattr__(name):
    if name == "binding":
        import importlib

        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
