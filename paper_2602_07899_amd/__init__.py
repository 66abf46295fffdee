"""MI355X-native TLQ scale-search hot path (HIP kernels behind a C ABI).

``paper_2602_07899_amd.tlq`` is the thin Python binding of ``libtlq.so``;
``paper_2602_07899_amd.workloads`` draws the seeded synthetic inputs.
Importing the package loads nothing native; the first call into ``tlq``
loads the shared library and raises if it has not been built.
"""
__all__ = ["tlq", "workloads"]
