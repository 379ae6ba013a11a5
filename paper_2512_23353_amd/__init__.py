"""MI355X-native ISOPO layer step (Gram -> coefficients -> weighted gradient).

`paper_2512_23353_amd.isopo` is the thin binding over the C-ABI library built
from `csrc/`; `paper_2512_23353_amd.workloads` draws the seeded synthetic
inputs.  Importing the package loads neither torch kernels nor the library;
the binding loads the library on first use and raises if it is not built.
"""
__all__ = ["isopo", "workloads"]
