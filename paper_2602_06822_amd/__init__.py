"""POP pruned-FFN hot path for MI355X: thin Python binding over the C-ABI HIP library.

`synth` (seeded input generators) imports without the library; everything else needs
`libpop_hip.so` built in-tree (`python -m paper_2602_06822_amd.build`) and raises if it is missing.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
