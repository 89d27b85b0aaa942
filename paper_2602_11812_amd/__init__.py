"""MI355X-native EGTP / PLP scoring (gfx950): thin Python binding over a C-ABI HIP library.

``workloads`` (seeded synthetic inputs) is importable without the library; everything in
``binding`` needs the built HIP library and fails loudly when it is missing.
"""
__all__ = ["binding", "workloads"]
