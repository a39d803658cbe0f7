"""MI355X-native Adasum tree combiner (arXiv 2006.02924, Sections 3-4).

``paper_2006_02924_amd.binding`` is the thin ctypes layer over the C-ABI
library ``libadasum.so`` (hand-written gfx950 HIP kernels);
``paper_2006_02924_amd.workloads`` makes seeded synthetic inputs.  There is no
CPU fallback: calling the binding without the built library raises.
"""
__version__ = "0.3.0"
