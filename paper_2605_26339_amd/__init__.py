"""QAM-W per-weight-matrix codec for MI355X (gfx950): hand-written HIP kernels behind a
C ABI (libqamw), with a thin ctypes binding.  `synth` holds the seeded input generators.

The binding is imported lazily so that `paper_2605_26339_amd.synth` can be used without
loading the HIP library.
"""
import importlib

__all__ = ["qamw", "synth"]


def __getattr__(name):
    if name in ("qamw", "synth"):
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
