"""MI355X-native BBMM inference hot path (arXiv 1809.11165).

`paper_1809_11165_amd.inputs`  -- seeded synthetic workloads (no method arithmetic)
`paper_1809_11165_amd.binding` -- ctypes binding over libbbmm.so (HIP, gfx950)

Nothing is imported eagerly: the binding loads the shared library on first use
and raises if it has not been built.
"""
__all__ = ["inputs", "binding"]
