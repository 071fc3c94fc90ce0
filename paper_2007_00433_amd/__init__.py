"""SESGD step library for AMD gfx950: Python binding over the C ABI in include/sesgd.h.

``workloads`` (shapes and seeded inputs) is importable without the HIP library; every
compute entry point lives in ``binding`` and raises if ``libsesgd.so`` is not built.
"""
__all__ = ["workloads", "binding", "build"]
