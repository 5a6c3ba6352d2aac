"""MI355X (gfx950) decode-step attention for TidalDecode (arxiv 2410.05076).

`paper_2410_05076_amd.tidal` is the thin ctypes binding over the C-ABI library
built from csrc/.  Nothing is loaded at import time; the HIP library is opened
on first use and its absence is an error, never a fallback.
"""
__all__ = ["tidal"]
