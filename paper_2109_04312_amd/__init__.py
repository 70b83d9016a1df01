"""MATE multi-view sparse attention (arXiv 2109.04312) for AMD MI355X (gfx950).

`paper_2109_04312_amd.mate`  -- thin ctypes binding over the C-ABI library (csrc/), which
                                holds every step of the path as hand-written HIP.
`paper_2109_04312_amd.synth` -- seeded synthetic inputs (no method arithmetic).

Nothing is imported eagerly: `synth` must stay usable without the built library.
"""
__all__ = ["mate", "synth"]
