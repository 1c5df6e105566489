"""PyramidKV prefill-time KV-cache compression for AMD MI355X (gfx950).

`paper_2406_02069_amd.binding` is the thin Python layer over the C-ABI library
libpkv (see include/pkv.h); `paper_2406_02069_amd.synth` holds the seeded
synthetic inputs.  Importing the package loads nothing native; the library is
loaded on first use and a missing library is an error, never a fallback.
"""
__all__ = ["binding", "synth", "build"]
