"""Token Recycling decode step for MI355X (gfx950).

`paper_2408_08696_amd.tr` is the thin binding over the C-ABI library built from
`csrc/`; `paper_2408_08696_amd.synth` produces seeded synthetic inputs.  Nothing is
imported eagerly so that the input generators stay usable without the library.
"""
__all__ = ["synth", "tr"]
