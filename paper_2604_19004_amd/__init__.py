"""Ocean SpGEMM hot path for AMD MI355X (gfx950).

``binding`` is the ctypes front end of the HIP library, ``build`` compiles it,
``workloads`` generates the seeded synthetic inputs.  Importing the package
does not need a GPU; calling into the library does.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding", "build"]
