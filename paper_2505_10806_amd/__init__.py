"""MI355X-native data path of RapidGNN: sampling, access histogram, hot-row cache, feature gather.

The compute lives in librapidgnn.so (hand-written HIP for gfx950, C ABI in include/rapidgnn.h);
``binding`` is the ctypes front end and ``pipeline`` drives an epoch (offline precompute + online
gather).  Import ``paper_2505_10806_amd.binding`` explicitly: it raises if the library is not built.
"""
__all__ = ["binding", "build", "pipeline"]
