"""MI355X-native hot path of feature whitening by gradient transformation (arXiv 2010.01546).

``paper_2010_01546_amd.binding`` is the thin ctypes layer over the C ABI declared in ``include/fw.h``;
``paper_2010_01546_amd.build`` compiles the HIP sources into ``libfw.so``.
"""
__all__ = ["binding", "build"]
