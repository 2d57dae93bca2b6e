"""Direct sparse convolution for MI355X (gfx950): Python face of the C-ABI library.

Importing the package loads nothing native.  `paper_1608_01409_amd.binding`
loads `libsconv.so` (built by `paper_1608_01409_amd.build`) on first use and
raises if it is missing: there is no CPU fallback.
"""

__all__ = ["binding", "build", "workloads"]
