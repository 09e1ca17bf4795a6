"""eOptShrinkQ KV-cache block compression for AMD MI355X (gfx950).

`paper_2605_02905_amd.eoq` is the thin ctypes binding of the C-ABI library built from
`csrc/`; `paper_2605_02905_amd.synth` generates the seeded synthetic workloads.
Importing the package loads nothing native; the first use of the binding does and
raises if the library has not been built.
"""
__all__ = ["eoq", "synth"]
