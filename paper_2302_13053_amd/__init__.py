"""MI355X-native embed-and-aggregate step of lazy message passing.

``binding`` mirrors the C ABI declared in ``include/retexo.h``; ``workloads``
draws the seeded synthetic inputs; ``build`` compiles the HIP library.
"""
from . import binding, workloads  # noqa: F401

__all__ = ["binding", "workloads"]
