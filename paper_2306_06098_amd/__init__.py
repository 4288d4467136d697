"""Sparse M-FAC / EFCP step for AMD MI355X (gfx950).

The compute lives in ``libefcp.so`` (hand-written HIP kernels behind a C ABI,
see ``include/efcp.h``); ``binding`` marshals arguments to it.  Importing this
package does not load the library; the first call does, and raises if the
library has not been built.
"""
__all__ = ["binding", "synth"]
