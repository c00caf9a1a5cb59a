"""Kunlun GDPA / sliding-window attention for MI355X (gfx950).

`workloads` (seeded input recipes) imports without the HIP library; `binding` loads
libkunlun.so and fails loudly if it has not been built.
"""
__all__ = ["workloads", "binding"]
