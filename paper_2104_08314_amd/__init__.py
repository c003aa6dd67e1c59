"""CPO / CPS sparse-activation convolution for AMD MI355X (arXiv 2104.08314).

``paper_2104_08314_amd.api`` is the binding of the C-ABI library (``include/cpoconv.h``);
``paper_2104_08314_amd.workloads`` generates the seeded synthetic layers; ``build`` compiles
the HIP sources.  Importing the package loads nothing: the library is opened on first use and
a missing library is an error, never a fallback.
"""

__all__ = ["api", "workloads", "build"]
