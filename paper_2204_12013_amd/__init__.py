"""Bamboo stage hot path for MI355X (gfx950).

`synth` holds the workload table and seeded inputs; `binding` is the thin
argument-marshalling layer over the C-ABI library `libbamboo_stage.so`
(imported lazily so that `synth` stays usable without the native library).
"""
from . import synth  # noqa: F401


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
