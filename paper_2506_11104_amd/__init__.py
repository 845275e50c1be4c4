"""MI355X-native hot path of DAM (Dynamic Attention Mask, arXiv 2506.11104).

``binding`` wraps the C-ABI library ``libdam.so`` (hand-written HIP for gfx950); ``workloads``
produces the seeded synthetic inputs. Importing the package does not load the library; the binding
does, and fails loudly when it has not been built.
"""
__all__ = ["binding", "workloads"]
