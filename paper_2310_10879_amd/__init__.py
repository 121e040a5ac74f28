"""BLoad block packer for MI355X (gfx950).

``paper_2310_10879_amd.bload`` is the binding over the C-ABI library (it needs the built
HIP library and raises if it is missing); ``paper_2310_10879_amd.workloads`` draws the
seeded synthetic inputs.  Nothing is imported eagerly so that the input
generators stay usable on a machine without the library.
"""

__all__ = ["bload", "workloads"]
