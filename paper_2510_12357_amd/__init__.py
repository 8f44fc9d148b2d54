"""MI355X-native hot path of the big-little MoE layer (MoBiLE, arXiv 2510.12357).

``workloads``  seeded synthetic layers (host buffers, numpy only)
``binding``    ctypes front end of the C-ABI library ``libmobile_moe.so`` (HIP, gfx950);
               importing it fails loudly when the library has not been built.
"""
__all__ = ["workloads"]
