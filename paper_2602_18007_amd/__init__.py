"""hxt: the per-GPU side of pipeline-parallel stage-boundary transfers on MI355X.

``paper_2602_18007_amd.hxt`` is the thin binding over the C-ABI library
(``libhxt.so``, hand-written HIP for gfx950); ``workloads`` describes the
synthetic messages.  Importing the package loads nothing native; the binding
raises if the library has not been built.
"""
__all__ = ["hxt", "workloads"]
