"""ST3 (Spatial-Temporal Visual Token Trimming) attention hot path for AMD MI355X.

`binding` mirrors include/st3.h over ctypes; `pipeline` issues those calls in the
order of the paper's Alg. 3.  Importing the package loads nothing; the shared
library is opened on first use and must have been built (`build.build_library()`).
"""
__all__ = ["binding", "pipeline", "build"]
