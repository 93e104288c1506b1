"""libtng on MI355X: the data-parallel hot path of Trajectory Normalized Gradients.

`paper_1901_08227_amd.binding` is the ctypes binding of the C-ABI library (HIP, gfx950);
`paper_1901_08227_amd.synth` draws the seeded synthetic inputs.  Importing the package
loads neither: the binding raises at first use when the built library is missing.
"""
__all__ = ["binding", "synth", "build"]
