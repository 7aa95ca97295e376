"""LASGD data-parallel hot path for MI355X (gfx950).

`workloads` is importable anywhere; `binding` loads the HIP shared library and
raises if it is missing (there is no CPU fallback on the product path).
"""
__all__ = ["workloads", "binding"]
