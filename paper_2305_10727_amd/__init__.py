"""gpusq: 2:4 structured-sparse FP16 / INT8 linear layers for AMD MI355X (gfx950).

The compute path lives in the C-ABI library built from csrc/ (hand-written HIP); `paper_2305_10727_amd.gpusq` is the thin ctypes
binding over it.  Importing the package loads nothing; the binding loads the library on first use and raises if
it has not been built.
"""
__all__ = ["gpusq", "synth"]
