"""Dynamic-batching data-parallel hot path for MI355X (gfx950).

`binding` wraps the C interface declared in include/dynb.h; `synth` holds the
seeded synthetic workloads.  The HIP library is loaded lazily by
`binding.load()`, which raises if it has not been built.
"""
__all__ = ["binding", "synth"]
